// Scale search for one output channel per workgroup without scoring every
// (element, candidate) pair.  Two kernels share the formulation below: sweep_sorted_kernel
// (first in this file) sorts the row and searches it; sweep_hist_kernel (second, with its own
// description) counts the row's bit patterns instead and is the one that runs wherever the
// clip ratios let its histogram fit, which includes the usual [0.5, 1].
//
// For a fixed scale the magnitude of the quantized value is a non-decreasing step function
// of the element's magnitude (rounding and the fp32 product are symmetric in the sign), so
// the elements that fall on one level magnitude form a contiguous run of the row sorted by
// magnitude.  The squared error of a candidate is then
//
//   sum (x - g s)^2 = sum x^2  -  2 s * sum_L |g_L| * S_L  +  s^2 * sum_L g_L^2 * n_L ,
//
// with S_L, n_L the sum of magnitudes and the count of the elements on the level pair +-g_L.
// INT4 is the one asymmetry: a negative element beyond -7.5 s lands on -8 where a positive
// one stays on 7; those elements (the negative ones past one more boundary) add their sum
// once more and 64 - 49 per element to the two level sums.  The kernel sorts the row once by
// magnitude (in-place LDS radix sort of the low 15 bits of the 16-bit patterns), builds
// prefix sums of the sorted magnitudes (and, sparser, of the negative elements' magnitudes
// and their number), and finds every level boundary of every candidate by binary search with
// the exact fp32 decision arithmetic (t = fl32(|x| * fl32(1/s)) against the rounding
// threshold of the boundary): 7 searches per candidate for E2M1, 8 for INT4.  That is
// O(n log n + K * levels * log n) per row instead of O(n * K).
//
// The formula cancels (the error is a few per cent of sum x^2), so it serves as a filter
// with a rigorous rounding bound: every candidate whose filtered error is within a wide
// margin of the smallest is shortlisted.  Where the shortlist of a format is one candidate
// and the bound is below 2^-34 of its filtered error, that value is the reported error.
// Otherwise (several candidates, exact ties, zero or tiny errors, non-finite input) the
// shortlist is re-scored element by element in fp64, exactly like the direct kernel, and
// the first smallest wins.
//
// Both apply to 16-bit inputs (fp16 / bf16) and the 4-bit formats (16 levels); other
// cases use the direct kernel in mofq_sweep.hip.
#include <cmath>
#include <type_traits>

#include "mofq_device.h"
#include "mofq_internal.h"

namespace mofq {

namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

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

// Padded position of sorted element i (in elements): a 2-element gap after every 64.
// Additive over sums of distinct powers of two, which the search below relies on.
MOFQ_DEV constexpr int phys(int i) { return i + ((i >> 6) << 1); }

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


template <typename In, int FA, int FB, int THREADS, int CH>
// second bound: waves per SIMD that the LDS footprint of the instance allows
__global__ __launch_bounds__(THREADS, (CH <= 4 ? 4 : 2)) void sweep_sorted_kernel(const SortedArgs a) {
  using L = Load8<In>;
  constexpr int NF = (FB >= 0) ? 2 : 1;
  constexpr int FBX = (FB >= 0) ? FB : FA;
  constexpr int NW = THREADS / 64;
  constexpr int E = CH * 8;            // keys per thread
  constexpr int NP = THREADS * E;      // padded row length
  constexpr int MAXL = NF * MOFQ_MAX_CLIP;

  // ---- LDS.  One key buffer, sorted in place (every pass holds all its keys in registers
  // before the first one is written back), and the digit counters.  The sorted row ends up in
  // a padded layout (one 4-byte gap after every 64 elements, so that the power-of-two strides
  // of a binary search do not all fall on one bank).  The counters then hold the prefix sums
  // (one exclusive prefix every BS positions).
  constexpr bool NP_POW2 = (NP & (NP - 1)) == 0;
  // first step of the boundary search; the padded row length is 2^k or 3 * 2^k
  constexpr int FIRST = NP_POW2 ? NP / 2 : NP / 3;
  static_assert((FIRST & (FIRST - 1)) == 0 && FIRST >= 64, "row length must be 2^k or 3 * 2^k");
  constexpr int LSTEPS = 32 - __builtin_clz(static_cast<unsigned>(FIRST));   // steps FIRST, FIRST/2, .., 1
  constexpr int KEYE = phys(NP) + 16;                      // elements of the key buffer (padded layout + slack)
  constexpr int KEYB = KEYE * 2;
  constexpr int CNTB = 16 * THREADS * 4 + 16;             // bytes of the digit counters (+ the last prefix)
  constexpr int BS = (8 * (NP / 2 + 1) <= CNTB) ? 2 : ((8 * (NP / 4 + 1) <= CNTB) ? 4 : 8);
  constexpr int NBLK = NP / BS;
  static_assert(8 * (NBLK + 1) <= CNTB, "prefix sums do not fit");
  static_assert(KEYB % 16 == 0, "the counters must stay 16-byte aligned");
  __shared__ __attribute__((aligned(16))) unsigned char s_raw[KEYB + CNTB];
  uint16_t* const s_keys = reinterpret_cast<uint16_t*>(s_raw);
  uint32_t (*const s_cnt)[THREADS] = reinterpret_cast<uint32_t (*)[THREADS]>(s_raw + KEYB);
  double* const s_blk = reinterpret_cast<double*>(s_raw + KEYB);   // [NBLK + 1], valid after the sort
  __shared__ uint32_t s_dig_tot[16];
  __shared__ float s_scale[NF][MOFQ_MAX_CLIP];
  __shared__ double s_fast[NF][MOFQ_MAX_CLIP];
  __shared__ float s_wmax[NW];
  __shared__ double s_wsum[3][NW];
  __shared__ double s_thr[NF];
  __shared__ int s_direct[NF];   // the winning candidate where no element-wise pass is needed, else -1
  __shared__ uint8_t s_list[MAXL];   // format * MOFQ_MAX_CLIP + candidate
  __shared__ int s_nlist;
  __shared__ double s_p2[NW];
  // re-scored errors of the shortlist: over the prefix sums, which are no longer needed by then
  double* const s_val = reinterpret_cast<double*>(s_raw + KEYB);
  static_assert(MAXL * 8 <= CNTB, "shortlist values do not fit");
  static_assert(MOFQ_MAX_CLIP * 2 <= 256, "shortlist entries are bytes");
  // INT4's negative elements beyond its last boundary: exclusive prefix of the negative elements'
  // magnitudes and of their number at every BSN-th position of the sorted row
  constexpr bool TAIL_A = FA == MOFQ_INT4, TAIL_B = (FB >= 0) && FBX == MOFQ_INT4;
  constexpr bool ANY_TAIL = TAIL_A || TAIL_B;
  constexpr int BSN = (THREADS == 256 && CH == 4) ? 32 : 16;   // what the LDS left beside the workgroups of a CU allows
  constexpr int NNEG = ANY_TAIL ? NP / BSN + 1 : 1;
  __shared__ double s_nsum[NNEG];
  __shared__ uint16_t s_ncnt[NNEG];
  __shared__ double s_wnsum[NW];
  __shared__ uint32_t s_wncnt[NW];
  static_assert(NP < 65536, "counts of negative elements are 16 bits");
  // Boundary search: with 16 waves the 8 boundaries of a candidate are dealt to SPLIT waves
  // (2 boundaries each) so that every wave has search work; the partial level sums meet in LDS.
  constexpr int SPLIT = (NW >= 16) ? 4 : 1;
  constexpr int NBD = 8;                  // 7 magnitude boundaries and INT4's extra one
  constexpr int QB = NBD / SPLIT;         // boundaries per lane
  static_assert(QB * SPLIT == NBD, "the boundaries must deal out evenly");
  __shared__ double s_pca[SPLIT > 1 ? NF * MOFQ_MAX_CLIP * SPLIT : 1];
  __shared__ int s_pcb[SPLIT > 1 ? NF * MOFQ_MAX_CLIP * SPLIT : 1];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint32_t tensor = 0;                                                    // wave-uniform
#pragma unroll
  for (int i = 1; i < kSweepGroupMax; ++i) tensor += (blockIdx.x >= a.row0[i]);
  const int64_t row = blockIdx.x - a.row0[tensor];
  const SortedTensor& T = a.t[tensor];
  const typename L::elem* src = static_cast<const typename L::elem*>(T.w) + row * T.ld;
  const int K = a.n_clip;
  const int n = static_cast<int>(a.cols);

  // ---- load the row: absmax, energy, and the sort keys ------------------------------
  float amax = 0.0f, l1f = 0.0f;
  uint32_t amax2 = 0;   // fp16 rows: running maximum of |x| in both halves of a register
  double en = 0.0;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int64_t c0 = (static_cast<int64_t>(j) * THREADS + tid) * 8;
    u32x4 raw = {0u, 0u, 0u, 0u};
    const bool ok = c0 < a.cols;
    if (ok) raw = *reinterpret_cast<const u32x4*>(src + c0);
    u32x4 keys;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t h0 = raw[i] & 0xFFFFu, h1 = raw[i] >> 16;
      const float v0 = bits_to_float<In>(h0), v1 = bits_to_float<In>(h1);
      if constexpr (std::is_same<In, F16>::value) {
        amax2 = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(f16x2, amax2),
                                                                       __builtin_bit_cast(f16x2, raw[i] & 0x7FFF7FFFu)));
      } else {
        amax = __builtin_fmaxf(amax, __builtin_fmaxf(__builtin_fabsf(v0), __builtin_fabsf(v1)));
      }
      const double d0 = static_cast<double>(v0), d1 = static_cast<double>(v1);
      en = __builtin_fma(d0, d0, en);
      en = __builtin_fma(d1, d1, en);
      l1f += __builtin_fabsf(v0) + __builtin_fabsf(v1);
      keys[i] = ok ? raw[i] : 0x7FFF7FFFu;   // padding: the largest magnitude pattern sorts last
    }
    *reinterpret_cast<u32x4*>(&s_keys[tid * E + j * 8]) = keys;
  }
  if constexpr (std::is_same<In, F16>::value)
    amax = __builtin_fmaxf(bits_to_float<In>(amax2 & 0xFFFFu), bits_to_float<In>(amax2 >> 16));
  amax = wave_max(amax);
  en = wave_sum(en);
  // sum |x| only enters the rounding bounds below: summed in fp32 (E + 7 additions of non-negative
  // terms, each off by at most 2^-24 relative; E <= 48) and raised by 2^-17 so that it stays an
  // upper bound
  double l1 = static_cast<double>(wave_sum_f32(l1f)) * (1.0 + 0x1p-17);
  if (lane == 0) { s_wmax[wave] = amax; s_wsum[0][wave] = en; s_wsum[1][wave] = l1; }
  __syncthreads();
  amax = s_wmax[0];
  en = s_wsum[0][0];
  l1 = s_wsum[1][0];
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    amax = __builtin_fmaxf(amax, s_wmax[w]);
    en += s_wsum[0][w];
    l1 += s_wsum[1][w];
  }
  for (int idx = tid; idx < NF * K; idx += THREADS) {
    const int f = idx / K, k = idx - f * K;
    const float qmax = (f == 0) ? Codec<FA>::QMAX : Codec<FBX>::QMAX;
    const float s = unit_scale(amax, a.clip[k], qmax, a.scale_f16 != 0);
    s_scale[f][k] = s;   // its reciprocal is taken where it is used: a table of them would cost a workgroup per compute unit
  }

  // ---- LSD radix sort by magnitude: digits of 4, 4, 4 and 3 bits of the low 15 bits of the
  // patterns; thread t owns positions [tE, tE+E).  LAST: the pass of the top digit, which writes
  // the patterns into the padded layout.
  auto radix_pass = [&](auto last_tag, const int shift) {
    constexpr bool LAST = decltype(last_tag)::value;
    constexpr int WIDTH = LAST ? 3 : 4;   // the sign bit is no part of the key
    constexpr int PER = THREADS / 64;   // counters of one digit per lane in the scan
    constexpr int DPW = 16 / NW;        // digits scanned by one wave
    constexpr int ND = 1 << WIDTH;      // digits that occur in this pass
#pragma unroll
    for (int d = 0; d < ND; ++d) s_cnt[d][tid] = 0;
    uint32_t kreg[E / 2];
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(&s_keys[tid * E + j * 8]);
#pragma unroll
      for (int i = 0; i < 4; ++i) kreg[j * 4 + i] = v[i];
    }
#pragma unroll
    for (int i = 0; i < E; ++i)   // own column: plain LDS add; positions are counted in bytes
      atomicAdd(&s_cnt[__builtin_amdgcn_ubfe(kreg[i >> 1], shift + (i & 1) * 16, WIDTH)][tid], 2u);
    __syncthreads();
    // per digit: exclusive scan of the counts across threads (kept in registers), digit totals aside
    uint32_t c[DPW][PER], base[DPW];
#pragma unroll
    for (int m = 0; m < DPW; ++m) {
      const int d = wave + m * NW;
      if (m * NW >= ND || d >= ND) continue;   // wave-uniform
      uint32_t sum = 0;
#pragma unroll
      for (int i = 0; i < PER; ++i) { c[m][i] = s_cnt[d][lane * PER + i]; sum += c[m][i]; }
      uint32_t total;
      base[m] = wave_excl_scan_u32(sum, total);
      if (lane == 0) s_dig_tot[d] = total;
    }
    __syncthreads();
    // start of each digit's run plus the scan: the first position of every (digit, thread)
    {
      // lane d of every wave: first position of digit d
      uint32_t unused;
      const uint32_t start = wave_excl_scan_u32(lane < ND ? s_dig_tot[lane & 15] : 0u, unused);
#pragma unroll
      for (int m = 0; m < DPW; ++m) {
        const int d = wave + m * NW;
        if (m * NW >= ND || d >= ND) continue;   // wave-uniform
        uint32_t bpos = base[m] + static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(start), d));
#pragma unroll
        for (int i = 0; i < PER; ++i) { s_cnt[d][lane * PER + i] = bpos; bpos += c[m][i]; }
      }
    }
    __syncthreads();
    uint32_t pos[E];
#pragma unroll
    for (int i = 0; i < E; ++i)   // stable: thread order, then i
      pos[i] = atomicAdd(&s_cnt[__builtin_amdgcn_ubfe(kreg[i >> 1], shift + (i & 1) * 16, WIDTH)][tid], 2u);
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const uint32_t v = (kreg[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu;
      // byte offset; the padded layout adds 4 bytes per 128
      const uint32_t off = LAST ? pos[i] + ((pos[i] >> 7) << 2) : pos[i];
      *reinterpret_cast<uint16_t*>(s_raw + off) = static_cast<uint16_t>(v);
    }
    __syncthreads();
  };
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) radix_pass(std::false_type{}, pass * 4);
  radix_pass(std::true_type{}, 12);
  // The buffer now holds the elements' own bit patterns in ascending order of magnitude.  Padding
  // is the pattern 0x7FFF (a NaN in fp16 and bf16), which fails every "<= threshold" test.
  const uint16_t* sorted = s_keys;       // padded layout: element i at sorted[phys(i)]

  // ---- prefix sums of the sorted magnitudes: exclusive prefix at every BS-th position; for INT4
  // also of the negative elements' magnitudes and of their number at every BSN-th position -------
  {
    constexpr int NB8 = 8 / BS;             // prefix entries per 8 elements
    constexpr int R8 = BSN / 8;             // 8-element pieces per entry of the negative elements' prefix
    double bs[CH][NB8], tsum = 0.0;
    double ng[CH], nsum = 0.0;
    uint32_t nc[CH], ncnt = 0;
    // no padding among this wave's positions: the common case needs no per-element test (the
    // second copy of the loop only pays where it is short)
    const bool wave_full = CH <= 4 && __builtin_amdgcn_readfirstlane((wave + 1) * 64 * E) <= n;
    // A wave whose largest magnitude stays below 7 on every candidate's INT4 scale holds no element
    // beyond INT4's last boundary (7.5 less one fp32 step) and neither does any wave before it:
    // their negative elements are left out of these prefixes (only differences between positions
    // at or beyond the first such element are ever taken) and their entries are never read.
    bool need_neg = false;
    if constexpr (ANY_TAIL) {
      constexpr int FT = TAIL_A ? 0 : 1;
      float s_min = __builtin_inff();
      for (int k = lane; k < K; k += 64) s_min = __builtin_fminf(s_min, s_scale[FT][k]);
      s_min = -wave_max(-s_min);
      const float inv_max = 1.0f / s_min;   // the largest reciprocal: the correctly rounded quotient does not increase with the scale
      const float x_hi = __builtin_fabsf(bits_to_float<In>(sorted[phys((wave + 1) * 64 * E - 1)]));
      need_neg = !(__builtin_amdgcn_readfirstlane(f2u(x_hi * inv_max)) < f2u(7.0f));   // non-negative floats order like their patterns; a NaN is above
    }
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const uint32_t* cp = reinterpret_cast<const uint32_t*>(&sorted[phys(tid * E + j * 8)]);
      const uint32_t v[4] = {cp[0], cp[1], cp[2], cp[3]};
#pragma unroll
      for (int g = 0; g < NB8; ++g) {
        double b = 0.0;
#pragma unroll
        for (int i = g * BS; i < (g + 1) * BS; ++i) {
          const uint32_t h = (v[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu;
          const int pos = tid * E + j * 8 + i;
          const double val = static_cast<double>(__builtin_fabsf(bits_to_float<In>(h)));
          b += (wave_full || pos < n) ? val : 0.0;
        }
        bs[j][g] = b;
        tsum += b;
      }
      ng[j] = 0.0;
      nc[j] = 0;
      if (need_neg) {   // wave-uniform; the padding pattern is positive
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t w = v[i] & sign_fill2(v[i]);   // positive halves become +0
          ng[j] += static_cast<double>(__builtin_fabsf(bits_to_float<In>(w & 0xFFFFu)));
          ng[j] += static_cast<double>(__builtin_fabsf(bits_to_float<In>(w >> 16)));
          nc[j] += static_cast<uint32_t>(__builtin_popcount(v[i] & 0x80008000u));
        }
        nsum += ng[j];
        ncnt += nc[j];
      }
    }
    double wtot;
    double base = wave_excl_scan_f64(tsum, wtot);
    double nbase = 0.0, wntot = 0.0;
    uint32_t cbase = 0, wctot = 0;
    if (need_neg) {
      nbase = wave_excl_scan_f64(nsum, wntot);
      cbase = wave_excl_scan_u32(ncnt, wctot);
    }
    if (lane == 0) { s_wsum[2][wave] = wtot; s_wnsum[wave] = wntot; s_wncnt[wave] = wctot; }
    __syncthreads();                       // also: every thread is done reading the sort buffers
    double wbase = 0.0;
    for (int w = 0; w < wave; ++w) wbase += s_wsum[2][w];
    base += wbase;
#pragma unroll
    for (int j = 0; j < CH; ++j)
#pragma unroll
      for (int g = 0; g < NB8; ++g) { s_blk[(tid * CH + j) * NB8 + g] = base; base += bs[j][g]; }
    if (tid == THREADS - 1) s_blk[NBLK] = base;
    if constexpr (ANY_TAIL) {
      if (need_neg || wave == NW - 1) {   // the last wave also leaves the totals
        for (int w = 0; w < wave; ++w) { nbase += s_wnsum[w]; cbase += s_wncnt[w]; }
#pragma unroll
        for (int j = 0; j < CH; ++j) {
          const int g8 = tid * CH + j;
          if (g8 % R8 == 0) { s_nsum[g8 / R8] = nbase; s_ncnt[g8 / R8] = static_cast<uint16_t>(cbase); }
          nbase += ng[j];
          cbase += nc[j];
        }
        if (tid == THREADS - 1) { s_nsum[NNEG - 1] = nbase; s_ncnt[NNEG - 1] = static_cast<uint16_t>(cbase); }
      }
    }
    __syncthreads();
  }
  const double s_total = s_blk[NBLK];

  // ---- level boundaries of every candidate by binary search ------------------------------
  // One lane per candidate (and per group of QB boundaries), one wave per (format, 64
  // candidates, boundary group); a lane walks the searches of its boundaries side by side
  // (independent chains hide the LDS latency) and adds up the two level sums itself.
  // Thresholds and level differences are wave-uniform.
  {
    // Lower bound over the first NP - 1 elements with the steps FIRST (twice when the row
    // length is 3 * 2^k), FIRST/2, .., 1: they add up to NP - 1 and no probe leaves that
    // range.  The last element is tested on its own afterwards.  Steps that are multiples of
    // 64 or distinct smaller powers of two keep the padded offsets additive.
    const uint32_t h_last = sorted[phys(NP - 1)];
    const uint32_t h_first = sorted[phys(FIRST - 1)];   // the first step's probe
    const int chunks = (K + 63) >> 6;
    // NQ: boundaries this lane searches; TAIL: the last of them is INT4's extra one
    auto unit = [&](auto nq_tag, auto tail_tag, const int f, const int k, const int sub) {
      constexpr int NQ = decltype(nq_tag)::value;
      constexpr bool TAIL = decltype(tail_tag)::value;
      const int q0 = sub * QB;                         // first boundary of this lane
      const float inv = 1.0f / s_scale[f][k < K ? k : K - 1];
      int ppos[NQ];   // padded byte offset of the next probe; of the position at the end
      // Branch-free: position = number of elements on level magnitudes <= m_q.  Every element
      // before the position passes the test; the NaN padding stops it at n.  The offset of the
      // next step's probe rides along in the position.  The first step probes the same element
      // for every boundary: one product serves them all.
      {
        constexpr int NEXT = NP_POW2 ? FIRST / 2 : FIRST;     // size of the step after the first
        const float t0 = scaled<In>(h_first, inv);
#pragma unroll
        for (int q = 0; q < NQ; ++q)
          ppos[q] = 2 * phys(NEXT - 1) + ((t0 <= a.thr[f][q0 + q]) ? 2 * phys(FIRST) : 0);
      }
#pragma unroll 1
      for (int st = (NP_POW2 ? LSTEPS - 2 : LSTEPS - 1); st >= 0; --st) {
        // wave-uniform constants of the step, computed on the scalar unit
        const int stp = 1 << __builtin_amdgcn_readfirstlane(st);
        const int next_probe = stp > 1 ? 2 * phys((stp >> 1) - 1) : 0;
        const int stay = next_probe - 2 * phys(stp - 1), go = stay + 2 * phys(stp);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          const uint32_t h = *reinterpret_cast<const uint16_t*>(s_raw + ppos[q]);
          const float t = scaled<In>(h, inv);
          ppos[q] += (t <= a.thr[f][q0 + q]) ? go : stay;
        }
      }
      const float t_last = scaled<In>(h_last, inv);
      double ca = 0.0;
      int cb4 = 0;       // 4 sum_b (count below boundary b) (m_b^2 - m_{b+1}^2): an integer below 2^31
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        // position in elements: the padded byte offset holds 132 bytes per 64 elements
        // (slot / 66 = slot * 993 >> 16 for every slot of a row of up to 24576 elements: the slot of
        // an element leaves a remainder of at most 63, so the quotient's fraction stays below 1 - 2/66
        // and the factor's excess of 5e-7 per slot cannot carry)
        const int slot = ppos[q] >> 1;
        const int j0 = slot - 2 * static_cast<int>(__umul24(static_cast<uint32_t>(slot), 993u) >> 16);
        const int j = j0 + (t_last <= a.thr[f][q0 + q] ? 1 : 0);
        if constexpr (TAIL) if (q == NQ - 1) {   // (the statement ends with `continue`)
          // negative elements at positions >= j: the totals less the prefix at j, which is the
          // entry of j's block plus the negative ones among the block's first j % BSN elements
          // (a block is 4-byte aligned and lies within one 64-element run of the padded layout)
          const int blk = j / BSN, rem = j % BSN;
          double pn = s_nsum[blk];
          uint32_t cn = s_ncnt[blk];
          // j = NP (rem = 0) reads nothing beyond the row: the addresses are clamped to the last block
          const uint32_t* bp = reinterpret_cast<const uint32_t*>(&sorted[phys((blk < NP / BSN ? blk : NP / BSN - 1) * BSN)]);
#pragma unroll
          for (int w = 0; w < BSN / 2; ++w) {
            uint32_t v = bp[w];
            v &= sign_fill2(v);                                   // negative elements only
            v &= (2 * w + 1 < rem) ? 0xFFFFFFFFu : ((2 * w < rem) ? 0x0000FFFFu : 0u);   // the first rem elements only
            pn += static_cast<double>(__builtin_fabsf(bits_to_float<In>(v & 0xFFFFu)));
            pn += static_cast<double>(__builtin_fabsf(bits_to_float<In>(v >> 16)));
            cn += static_cast<uint32_t>(__builtin_popcount(v & 0x80008000u));
          }
          ca = __builtin_fma(s_nsum[NNEG - 1] - pn, a.dgd[f][q0 + q], ca);
          cb4 = __mul24(static_cast<int>(s_ncnt[NNEG - 1]) - static_cast<int>(cn), a.dg2q[f][q0 + q]) + cb4;
          continue;
        }
        {
          constexpr int LB = (BS == 2) ? 1 : (BS == 4 ? 2 : 3);
          double p = s_blk[j >> LB];
          if constexpr (BS == 2) {
            // an odd position adds the element before it, which sits at the offset rounded down
            // to 4 bytes (an even position reads its own element there and drops it; j = NP is even)
            const uint32_t hv = *reinterpret_cast<const uint16_t*>(s_raw + (ppos[q] & ~3));
            p += static_cast<double>(__builtin_fabsf(bits_to_float<In>(hv & static_cast<uint32_t>(-(j & 1)))));
          } else {
            const int jb = phys(j & ~(BS - 1));
#pragma unroll
            for (int i = 0; i < BS - 1; ++i) {
              const bool in = i < (j & (BS - 1));
              const double val = static_cast<double>(__builtin_fabsf(bits_to_float<In>(sorted[in ? jb + i : 0])));
              p += in ? val : 0.0;
            }
          }
          ca = __builtin_fma(p, a.dgd[f][q0 + q], ca);
          cb4 = __mul24(j, a.dg2q[f][q0 + q]) + cb4;
        }
      }
      if constexpr (SPLIT == 1) {
        if (k < K) {
          const double gl = static_cast<double>(a.g_last[f]);
          const double A = ca + gl * s_total;
          const double B = 0.25 * static_cast<double>(cb4) + gl * gl * static_cast<double>(n);
          const double sc = static_cast<double>(s_scale[f][k]);
          s_fast[f][k] = (en - 2.0 * sc * A) + sc * sc * B;   // filtered error
        }
      } else {
        if (k < K) {
          s_pca[(f * MOFQ_MAX_CLIP + k) * SPLIT + sub] = ca;
          s_pcb[(f * MOFQ_MAX_CLIP + k) * SPLIT + sub] = cb4;
        }
      }
    };
    for (int u = wave; u < NF * chunks * SPLIT; u += NW) {
      const int sub = u % SPLIT, fc = u / SPLIT;      // wave-uniform
      const int f = fc / chunks;
      const int k = (fc - f * chunks) * 64 + lane;
      const bool tail = (f == 0) ? TAIL_A : TAIL_B;   // wave-uniform
      if constexpr (SPLIT == 1) {
        if (tail) unit(std::integral_constant<int, 8>{}, std::true_type{}, f, k, sub);
        else unit(std::integral_constant<int, 7>{}, std::false_type{}, f, k, sub);
      } else {
        // E2M1's slot 7 carries zero weights and a threshold no element passes
        if (tail && sub == SPLIT - 1) unit(std::integral_constant<int, QB>{}, std::true_type{}, f, k, sub);
        else unit(std::integral_constant<int, QB>{}, std::false_type{}, f, k, sub);
      }
    }
    if constexpr (SPLIT > 1) {
      __syncthreads();
      for (int idx = tid; idx < NF * K; idx += THREADS) {
        const int f = idx / K, k = idx - f * K;
        double ca = 0.0;
        int cb4 = 0;
#pragma unroll
        for (int sub = 0; sub < SPLIT; ++sub) {   // fixed order
          ca += s_pca[(f * MOFQ_MAX_CLIP + k) * SPLIT + sub];
          cb4 += s_pcb[(f * MOFQ_MAX_CLIP + k) * SPLIT + sub];
        }
        const double gl = static_cast<double>(a.g_last[f]);
        const double A = ca + gl * s_total;
        const double B = 0.25 * static_cast<double>(cb4) + gl * gl * static_cast<double>(n);
        const double sc = static_cast<double>(s_scale[f][k]);
        s_fast[f][k] = (en - 2.0 * sc * A) + sc * sc * B;   // filtered error
      }
    }
  }
  __syncthreads();

  // ---- shortlist: candidates the filter cannot separate from the best ---------------------
  // Rounding of the filtered error, with u = 2^-53.  Every prefix sum (of magnitudes: no
  // cancellation) comes from a summation tree of depth at most D = 2E + 32 (thread-sequential,
  // wave scan, across waves, the elements of a partly covered block) and is off by at most
  // D u sum|x|; the level differences of one format add up to at most 7, the largest level of
  // the symmetric part is at most 7 and INT4's extra level adds the difference of two such
  // prefix sums once, so the level sum A is off by less than 32 D u sum|x| including its own
  // additions (8, and 3 more where the boundaries are dealt to four waves).  The energy is off
  // by (E + 14) u sum x^2; counts, level squares and
  // s^2 are exact; the remaining products and additions round a handful of times on terms
  // bounded by the three summands.  Hence
  //   |filtered - exact| <= beta = u (40 D * 2 s sum|x| + (E + 32) sum x^2 + 8 s^2 g_max^2 n).
  // The shortlist margin is far wider: 2^-33 of sum x^2 + 2 s g_max sum|x| + s^2 g_max^2 n.
  // A format whose shortlist is a single candidate has its winner already; when beta is below
  // 2^-34 of that candidate's filtered error, the filtered error is reported as it stands and
  // the element-wise pass is skipped for the format.
  for (int f = wave; f < NF; f += NW) {
    double m = __builtin_inf();
    int km = 0;
    float smax = 0.0f;
    for (int k = lane; k < K; k += 64) {
      const double v = s_fast[f][k];
      if (v < m) { m = v; km = k; }
      smax = __builtin_fmaxf(smax, s_scale[f][k]);
    }
    wave_argmin(m, km);
    smax = wave_max(smax);
    const double sm = static_cast<double>(smax), gm = static_cast<double>(a.g_absmax[f]);
    const double nd = static_cast<double>(n);
    const double mag = en + 2.0 * sm * gm * l1 + sm * sm * gm * gm * nd;
    const double thr = m + 0x1p-33 * mag;   // twice the margin: both values carry the error
    int cnt = 0;
    for (int k0 = 0; k0 < K; k0 += 64) {
      const int k = k0 + lane;
      cnt += __builtin_popcountll(__ballot(k < K && !(s_fast[f][k < K ? k : 0] > thr)));
    }
    const double beta = 0x1p-53 * (40.0 * (2 * E + 32) * 2.0 * sm * l1 + (E + 32) * en + 8.0 * sm * sm * gm * gm * nd);
    const bool direct = cnt == 1 && beta <= 0x1p-34 * m;   // false for a zero or non-finite error
    if (lane == 0) { s_thr[f] = thr; s_direct[f] = direct ? km : -1; }
  }
  if (tid == 0) s_nlist = 0;
  __syncthreads();
  for (int idx = tid; idx < NF * K; idx += THREADS) {
    const int f = idx / K, k = idx - f * K;
    if (s_direct[f] < 0 && !(s_fast[f][k] > s_thr[f]))
      s_list[atomicAdd(&s_nlist, 1)] = static_cast<uint8_t>(f * MOFQ_MAX_CLIP + k);   // any order
  }
  __syncthreads();
  const int n_list = s_nlist;

  // ---- exact fp64 re-score of the shortlist, element by element (sorted order) ------------
  uint32_t carry = 0;
  for (int e = 0; e < n_list; ++e) {
    const int fk = s_list[e];
    const int f = __builtin_amdgcn_readfirstlane(fk / MOFQ_MAX_CLIP);
    const int k = __builtin_amdgcn_readfirstlane(fk % MOFQ_MAX_CLIP);
    const float s = s_scale[f][k], inv = 1.0f / s;
    const double sd = static_cast<double>(s);
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const int p0 = tid * E + j * 8;
      if (__builtin_amdgcn_readfirstlane(wave * 64 * E + j * 8) < n) {   // wave-uniform: any data here?
        const uint32_t* cp = reinterpret_cast<const uint32_t*>(&sorted[phys(p0)]);
        const uint32_t v[4] = {cp[0], cp[1], cp[2], cp[3]};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float x0 = (p0 + 2 * i < n) ? bits_to_float<In>(v[i] & 0xFFFFu) : 0.0f;
          const float x1 = (p0 + 2 * i + 1 < n) ? bits_to_float<In>(v[i] >> 16) : 0.0f;
          if (f == 0) rescore2<FA>(acc, x0, x1, inv, sd, carry);
          else rescore2<FBX>(acc, x0, x1, inv, sd, carry);
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

  if (tid < NF) {
    const int f = tid;
    double best = __builtin_inf();
    int bk = s_direct[f];
    if (bk >= 0) best = s_fast[f][bk];
    for (int e = 0; e < n_list; ++e) {   // smallest error, then smallest index: the first smallest
      const int fk = s_list[e];
      if (fk / MOFQ_MAX_CLIP != f) continue;
      const int k = fk % MOFQ_MAX_CLIP;
      if (s_val[e] < best || (s_val[e] == best && k < bk)) { best = s_val[e]; bk = k; }
    }
    if (bk < 0) { bk = 0; best = __builtin_nan(""); }   // only on non-finite input
    T.rec.scale[f][row] = s_scale[f][bk];
    T.rec.clip[f][row] = bk;
    T.rec.err[f][row] = best;
    if (f == 0 && T.rec.energy) T.rec.energy[row] = en;
  }
}

// ---- the same search from a histogram of the magnitudes' bit patterns --------------------------
//
// The decision "fl32(|x| * inv) <= threshold" is monotone in the magnitude's bit pattern, so for
// every (candidate, boundary) there is one largest pattern H that passes, and the elements on
// level magnitudes up to m_b are those with pattern <= H.  Instead of sorting the row, the kernel
// counts the elements per pattern (16-bit counters, two per word, LDS adds), forms count and
// magnitude-sum prefixes over groups of 8 patterns (a group shares its exponent, so its elements'
// magnitudes are v0 + i ulp and its sum is v0 C + ulp sum i c_i, exact in fp64), finds H from
// an fp32 estimate proven with two exact decisions (a pattern-space binary search where the
// estimate is off), and reads count and sum up to H from the group
// prefix and one 16-byte read of the group's counters.  Only the patterns between the smallest
// threshold and the row's largest magnitude get a counter: elements below every threshold sit on
// level 0 for every candidate and drop out of both level sums.  How many patterns that is
// depends on the clip ratios alone, so the host sizes the histogram (dynamic LDS) and uses the
// sorting kernel where it would not fit.  INT4's negative elements beyond its extra boundary
// are counted in a second, short histogram over the top of the range.
//
// Filter, shortlist and exact fp64 re-score are those of the sorting kernel; the re-score reads
// the row again.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
MOFQ_DEV uint32_t dot2(uint32_t a, uint32_t b, uint32_t c) {   // a.lo b.lo + a.hi b.hi + c
  return __builtin_amdgcn_udot2(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b), c, false);
}

MOFQ_DEV int med3i(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }   // x clamped to [lo, hi]

// bit pattern of x >= 0 rounded toward zero to the input type; largest finite pattern
template <typename In> MOFQ_DEV uint32_t pattern_rtz(float x);
template <> MOFQ_DEV uint32_t pattern_rtz<F16>(float x) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(x, 0.0f)) & 0xFFFFu;
}
template <> MOFQ_DEV uint32_t pattern_rtz<BF16>(float x) { return f2u(x) >> 16; }
template <typename In> struct Pattern;
template <> struct Pattern<F16> { static constexpr int MAX_FINITE = 0x7BFF; };
template <> struct Pattern<BF16> { static constexpr int MAX_FINITE = 0x7F7F; };

// Lexicographic minimum of (value, index) over the wave by data-parallel-primitive moves: the
// smallest value (no NaN among the inputs), then the smallest index among the lanes that hold it.
template <int CTRL> MOFQ_DEV int dpp_i32(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, true); }
MOFQ_DEV void wave_argmin_dpp(double& v, int& idx) {
  double m = v;
  m = __builtin_fmin(m, dpp_f64<DPP_QUAD_XOR1>(m));
  m = __builtin_fmin(m, dpp_f64<DPP_QUAD_XOR2>(m));
  m = __builtin_fmin(m, dpp_f64<DPP_ROW_HALF_MIRROR>(m));
  m = __builtin_fmin(m, dpp_f64<DPP_ROW_MIRROR>(m));
  m = __builtin_fmin(__builtin_fmin(readlane_f64(m, 0), readlane_f64(m, 16)), __builtin_fmin(readlane_f64(m, 32), readlane_f64(m, 48)));
  int c = (v == m) ? idx : 0x7FFFFFFF;
  c = min(c, dpp_i32<DPP_QUAD_XOR1>(c));
  c = min(c, dpp_i32<DPP_QUAD_XOR2>(c));
  c = min(c, dpp_i32<DPP_ROW_HALF_MIRROR>(c));
  c = min(c, dpp_i32<DPP_ROW_MIRROR>(c));
  idx = min(min(__builtin_amdgcn_readlane(c, 0), __builtin_amdgcn_readlane(c, 16)),
            min(__builtin_amdgcn_readlane(c, 32), __builtin_amdgcn_readlane(c, 48)));
  v = m;
}

constexpr int kHistMaxBins = 8192;      // patterns with a counter (16 KB)
constexpr int kHistMaxTailBins = 2048;  // of INT4's negative elements

// Count and magnitude sum of the elements in the histogram's first n1 counters, 0 <= n1 <= nbin:
// the exclusive prefixes of group n1 / 8 plus the first n1 % 8 counters of that group (n1 = nbin
// reads the 16 bytes after the counters, which are inside the workgroup's LDS, and masks them all).
// hist: counters, two per word; cntp / sump: exclusive prefixes per group of 8 counters;
// keep[c]: masks of the first c of a group's eight counters (a table in LDS: one read instead of
// sixteen compare-and-select instructions).
template <typename In>
MOFQ_DEV void hist_prefix(const uint32_t* hist, const uint16_t* cntp, const double* sump, const u32x4* keep, int lo,
                          int n1, uint32_t& C, double& S) {
  const int g = n1 >> 3;
  const u32x4 w = *reinterpret_cast<const u32x4*>(hist + 4 * g);
  const u32x4 m = keep[n1 & 7];   // 16-bit masks, two per word
  uint32_t cin = 0, win = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t v = w[i] & m[i];
    cin = dot2(v, 0x00010001u, cin);
    win = dot2(v, static_cast<uint32_t>(2 * i) | (static_cast<uint32_t>(2 * i + 1) << 16), win);
  }
  const float v0 = bits_to_float<In>(static_cast<uint32_t>(lo + 8 * g));
  const float ulp = bits_to_float<In>(static_cast<uint32_t>(lo + 8 * g + 1)) - v0;   // exact
  double s = sump[g];
  s = __builtin_fma(static_cast<double>(v0), static_cast<double>(cin), s);
  s = __builtin_fma(static_cast<double>(ulp), static_cast<double>(win), s);
  C = cntp[g] + cin;
  S = s;
}

// Exclusive prefixes of count and magnitude sum per group of 8 bins; the totals in entry ng.
// Thread t takes the groups [t gp, (t + 1) gp), gp <= GPMAX.  Called by all threads.
template <typename In, int THREADS, int GPMAX>
MOFQ_DEV void hist_group_prefixes(const uint32_t* hist, uint16_t* cntp, double* sump, int lo, int ng, int gp,
                                  uint32_t* s_wc, double* s_ws) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t c8[GPMAX];
  double s8[GPMAX];
  uint32_t ct = 0;
  double st = 0.0;
#pragma unroll
  for (int i = 0; i < GPMAX; ++i) {
    const int g = tid * gp + i;
    c8[i] = 0;
    s8[i] = 0.0;
    if (i < gp && g < ng) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(hist + 4 * g);
      uint32_t c = 0, wsum = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c = dot2(w[j], 0x00010001u, c);
        wsum = dot2(w[j], static_cast<uint32_t>(2 * j) | (static_cast<uint32_t>(2 * j + 1) << 16), wsum);
      }
      const float v0 = bits_to_float<In>(static_cast<uint32_t>(lo + 8 * g));
      const float ulp = bits_to_float<In>(static_cast<uint32_t>(lo + 8 * g + 1)) - v0;
      c8[i] = c;
      s8[i] = __builtin_fma(static_cast<double>(ulp), static_cast<double>(wsum), static_cast<double>(v0) * static_cast<double>(c));
      ct += c;
      st += s8[i];
    }
  }
  uint32_t wct;
  double wst;
  uint32_t cb = wave_excl_scan_u32(ct, wct);
  double sb = wave_excl_scan_f64(st, wst);
  if (lane == 0) { s_wc[wave] = wct; s_ws[wave] = wst; }
  __syncthreads();
  for (int w = 0; w < wave; ++w) { cb += s_wc[w]; sb += s_ws[w]; }
#pragma unroll
  for (int i = 0; i < GPMAX; ++i) {
    const int g = tid * gp + i;
    if (i < gp && g < ng) { cntp[g] = static_cast<uint16_t>(cb); sump[g] = sb; }
    cb += c8[i];
    sb += s8[i];
  }
  if (tid == THREADS - 1) { cntp[ng] = static_cast<uint16_t>(cb); sump[ng] = sb; }
  __syncthreads();
}

// The same for a short histogram (at most 64 * GPMAX groups) by one wave alone, without barriers:
// lane l takes the groups [l gp, (l + 1) gp).  The caller's next barrier publishes the result.
template <typename In, int GPMAX>
MOFQ_DEV void hist_group_prefixes_wave(const uint32_t* hist, uint16_t* cntp, double* sump, int lo, int ng, int gp) {
  const int lane = threadIdx.x & 63;
  uint32_t c8[GPMAX];
  double s8[GPMAX];
  uint32_t ct = 0;
  double st = 0.0;
#pragma unroll
  for (int i = 0; i < GPMAX; ++i) {
    const int g = lane * gp + i;
    c8[i] = 0;
    s8[i] = 0.0;
    if (i < gp && g < ng) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(hist + 4 * g);
      uint32_t c = 0, wsum = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c = dot2(w[j], 0x00010001u, c);
        wsum = dot2(w[j], static_cast<uint32_t>(2 * j) | (static_cast<uint32_t>(2 * j + 1) << 16), wsum);
      }
      const float v0 = bits_to_float<In>(static_cast<uint32_t>(lo + 8 * g));
      const float ulp = bits_to_float<In>(static_cast<uint32_t>(lo + 8 * g + 1)) - v0;
      c8[i] = c;
      s8[i] = __builtin_fma(static_cast<double>(ulp), static_cast<double>(wsum), static_cast<double>(v0) * static_cast<double>(c));
      ct += c;
      st += s8[i];
    }
  }
  uint32_t wct;
  double wst;
  uint32_t cb = wave_excl_scan_u32(ct, wct);
  double sb = wave_excl_scan_f64(st, wst);
#pragma unroll
  for (int i = 0; i < GPMAX; ++i) {
    const int g = lane * gp + i;
    if (i < gp && g < ng) { cntp[g] = static_cast<uint16_t>(cb); sump[g] = sb; }
    cb += c8[i];
    sb += s8[i];
  }
  if (lane == 63) { cntp[ng] = static_cast<uint16_t>(cb); sump[ng] = sb; }
}

template <typename In, int FA, int FB, int CH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(CH <= 2 ? 5 : (CH <= 6 ? 4 : 3))))
void sweep_hist_kernel(const SortedArgs a) {
  using L = Load8<In>;
  constexpr int THREADS = 256;
  constexpr int NF = (FB >= 0) ? 2 : 1;
  constexpr int FBX = (FB >= 0) ? FB : FA;
  constexpr int NW = THREADS / 64;
  constexpr int E = CH * 8;            // elements per thread
  constexpr int MAXL = NF * MOFQ_MAX_CLIP;
  constexpr bool TAIL_A = FA == MOFQ_INT4, TAIL_B = (FB >= 0) && FBX == MOFQ_INT4;
  constexpr bool ANY_TAIL = TAIL_A || TAIL_B;
  constexpr int GPMAX = kHistMaxBins / 8 / THREADS;   // groups per thread at most

  // dynamic LDS: [sump | tsump | hist | thist | cntp | tcntp]
  extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
  const int nbin = a.nbin, ntbin = ANY_TAIL ? a.ntbin : 0;   // multiples of 8
  const int ng = nbin >> 3, ntg = ntbin >> 3;
  double* const sump = reinterpret_cast<double*>(s_dyn);
  double* const tsump = sump + (ng + 1);
  uint32_t* const hist = reinterpret_cast<uint32_t*>(s_dyn + (((ng + 1) + (ntg + 1)) * 8 + 15) / 16 * 16);
  uint32_t* const thist = hist + (nbin >> 1);
  uint16_t* const cntp = reinterpret_cast<uint16_t*>(thist + (ntbin >> 1));   // counts stay below 2^16: a row has at most 24576 elements
  uint16_t* const tcntp = cntp + (ng + 1);

  __shared__ float s_scale[NF][MOFQ_MAX_CLIP];
  __shared__ double s_fast[NF][MOFQ_MAX_CLIP];
  __shared__ float s_wmax[NW];
  __shared__ double s_wsum[1][NW];
  __shared__ uint32_t s_wc[NW];
  __shared__ double s_ws[NW];
  __shared__ double s_thr[NF];
  __shared__ int s_direct[NF];   // the winning candidate where no element-wise pass is needed, else -1
  __shared__ uint8_t s_list[MAXL];   // format * MOFQ_MAX_CLIP + candidate
  __shared__ int s_nlist;
  __shared__ double s_p2[NW];
  // re-scored errors of the shortlist: over the sum prefixes, which are no longer needed by then
  // (the host sizes the dynamic LDS for it)
  double* const s_val = reinterpret_cast<double*>(s_dyn);
  __shared__ __attribute__((aligned(16))) uint32_t s_keep[8][4];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint32_t tensor = 0;                                                    // wave-uniform
#pragma unroll
  for (int i = 1; i < kSweepGroupMax; ++i) tensor += (blockIdx.x >= a.row0[i]);
  const int64_t row = blockIdx.x - a.row0[tensor];
  const SortedTensor& T = a.t[tensor];
  const typename L::elem* src = static_cast<const typename L::elem*>(T.w) + row * T.ld;
  const int K = a.n_clip;
  const int n = static_cast<int>(a.cols);
  if (tid < 32) {   // word tid % 4 of the mask of the first tid / 4 counters
    const int c = tid >> 2, i = tid & 3;
    s_keep[c][i] = (c >= 2 * i + 2) ? 0xFFFFFFFFu : ((c == 2 * i + 1) ? 0x0000FFFFu : 0u);
  }
  const u32x4* const keep = reinterpret_cast<const u32x4*>(&s_keep[0][0]);

  // ---- load the row (it stays in registers until it is counted): absmax, energy; clear the counters ---
  u32x4 rawv[CH];
  float amax = 0.0f;
  uint32_t amax2 = 0;   // fp16 rows: running maximum of |x| in both halves of a register
  double en = 0.0;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int64_t c0 = (static_cast<int64_t>(j) * THREADS + tid) * 8;
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (c0 < a.cols) raw = *reinterpret_cast<const u32x4*>(src + c0);
    rawv[j] = raw;
  }
  {
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int i = tid; i < ng + ntg; i += THREADS) reinterpret_cast<u32x4*>(hist)[i] = zero;   // hist and thist are adjacent
  }
#pragma unroll
  for (int j = 0; j < CH; ++j) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t h0 = rawv[j][i] & 0xFFFFu, h1 = rawv[j][i] >> 16;
      const float v0 = bits_to_float<In>(h0), v1 = bits_to_float<In>(h1);
      if constexpr (std::is_same<In, F16>::value) {
        amax2 = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(f16x2, amax2),
                                                                       __builtin_bit_cast(f16x2, rawv[j][i] & 0x7FFF7FFFu)));
      } else {
        amax = __builtin_fmaxf(amax, __builtin_fmaxf(__builtin_fabsf(v0), __builtin_fabsf(v1)));
      }
      const double d0 = static_cast<double>(v0), d1 = static_cast<double>(v1);
      en = __builtin_fma(d0, d0, en);
      en = __builtin_fma(d1, d1, en);
    }
  }
  if constexpr (std::is_same<In, F16>::value)
    amax = __builtin_fmaxf(bits_to_float<In>(amax2 & 0xFFFFu), bits_to_float<In>(amax2 >> 16));
  amax = wave_max(amax);
  en = wave_sum(en);
  if (lane == 0) { s_wmax[wave] = amax; s_wsum[0][wave] = en; }
  __syncthreads();   // also: the counters are clear
  amax = s_wmax[0];
  en = s_wsum[0][0];
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    amax = __builtin_fmaxf(amax, s_wmax[w]);
    en += s_wsum[0][w];
  }
  if (tid < 2 * MOFQ_MAX_CLIP) {   // thread f * MOFQ_MAX_CLIP + k
    const int f = tid / MOFQ_MAX_CLIP, k = tid % MOFQ_MAX_CLIP;
    const float qmax = (f == 0) ? Codec<FA>::QMAX : Codec<FBX>::QMAX;
    if (f < NF && k < K) s_scale[f][k] = unit_scale(amax, a.clip[k], qmax, a.scale_f16 != 0);
  }
  static_assert(2 * MOFQ_MAX_CLIP <= THREADS, "one thread per (format, candidate)");

  // ---- the histogram covers the nbin patterns up to the largest magnitude's (a non-finite
  // element lands in the last counter: the row's error is non-finite anyway) --------------------
  const int hmax = static_cast<int>(pattern_rtz<In>(amax < 3.0e38f ? amax : 3.0e38f));   // exact for a finite amax
  const int lo = (((hmax + 1 - nbin) > 0 ? (hmax + 1 - nbin) : 0) + 7) & ~7;
  const int tlo = (((hmax + 1 - ntbin) > 0 ? (hmax + 1 - ntbin) : 0) + 7) & ~7;
  {
    // both halves of a word at once: signed 16-bit differences to the first counted pattern
    // (patterns are below 2^15), clamped to the last counter
    const i16x2 lo2 = {static_cast<short>(lo), static_cast<short>(lo)};
    const i16x2 tlo2 = {static_cast<short>(tlo), static_cast<short>(tlo)};
    const i16x2 last2 = {static_cast<short>(nbin - 1), static_cast<short>(nbin - 1)};
    const i16x2 tlast2 = {static_cast<short>(ntbin - 1), static_cast<short>(ntbin - 1)};
    auto count = [](uint32_t* h, int b) { atomicAdd(&h[b >> 1], 1u << ((b & 1) * 16)); };
#pragma unroll
    for (int j = 0; j < CH; ++j) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t w = rawv[j][i];
        const i16x2 h2 = __builtin_bit_cast(i16x2, w & 0x7FFF7FFFu);
        const i16x2 b2 = __builtin_elementwise_min(h2 - lo2, last2);
        // padding (zero) and whatever lies below every threshold has no counter
        if (b2[0] >= 0) count(hist, b2[0]);
        if (b2[1] >= 0) count(hist, b2[1]);
        if constexpr (ANY_TAIL) {
          const i16x2 t2 = h2 - tlo2;
          // halves that are negative elements at or above the short histogram's first pattern
          const uint32_t q2 = sign_fill2(w) & ~sign_fill2(__builtin_bit_cast(uint32_t, t2));
          if (q2 != 0) {
            const i16x2 tc2 = __builtin_elementwise_min(t2, tlast2);
            if (q2 & 0xFFFFu) count(thist, tc2[0]);
            if (q2 >> 16) count(thist, tc2[1]);
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- group prefixes ----------------------------------------------------------------------------
  // (the short histogram by the last wave alone, before the barriers of the long one's prefixes)
  if constexpr (ANY_TAIL)
    if (wave == NW - 1) hist_group_prefixes_wave<In, kHistMaxTailBins / 8 / 64>(thist, tcntp, tsump, tlo, ntg, (ntg + 63) / 64);
  hist_group_prefixes<In, THREADS, GPMAX>(hist, cntp, sump, lo, ng, (ng + THREADS - 1) / THREADS, s_wc, s_ws);
  const uint32_t c_total = cntp[ng];
  const double s_total = sump[ng];
  // sum |x| enters the rounding bounds only: the counted elements' sum (raised beyond its rounding)
  // plus, for every other element, the magnitude of the first counted pattern, which exceeds its own
  const double l1 = s_total * (1.0 + 0x1p-40) + static_cast<double>(n) * static_cast<double>(bits_to_float<In>(static_cast<uint32_t>(lo)));

  // ---- level boundaries of every candidate: one lane per candidate, one wave per (format, 64
  // candidates) --------------------------------------------------------------------------------
  {
    const int chunks = (K + 63) >> 6;
    auto unit = [&](auto tail_tag, const int f, const int k) {
      constexpr bool TAIL = decltype(tail_tag)::value;
      const float s = s_scale[f][k < K ? k : K - 1];
      const float inv = 1.0f / s;
      // H = the largest finite pattern h with fl32(v(h) * inv) <= thr.  v(0) = 0 passes.
      auto threshold_pattern = [&](const float thr) {
        auto pass = [&](int h) { return scaled<In>(static_cast<uint32_t>(h), inv) <= thr; };
        // estimate: the pattern of thr * s rounded toward zero, which is H unless a pattern's
        // value lies in the gap of a few fp32 steps between that product and the real boundary
        int H = static_cast<int>(pattern_rtz<In>(thr * s));
        H = H > Pattern<In>::MAX_FINITE - 1 ? Pattern<In>::MAX_FINITE - 1 : H;
        const bool at = pass(H), above = pass(H + 1);   // both always: a short circuit costs more than it saves
        if (!(static_cast<int>(at) & static_cast<int>(!above))) {   // (also: no finite pattern fails)
          int lo_h = 0, hi_h = Pattern<In>::MAX_FINITE;   // pass(lo_h) holds; the answer is in [lo_h, hi_h]
          while (lo_h < hi_h) {
            const int mid = (lo_h + hi_h + 1) >> 1;
            if (pass(mid)) lo_h = mid;
            else hi_h = mid - 1;
          }
          H = lo_h;
        }
        return H;
      };
      double ca = 0.0;
      int cb4 = 0;       // 4 sum_b (count up to boundary b) (m_b^2 - m_{b+1}^2): an integer below 2^31
      // counters at or below H, as a number of counters: H - lo + 1 within [0, nbin].  A threshold
      // more than one pattern below the histogram's range (least < 0) sends the candidate to the
      // exact pass: uncounted elements might lie above it.
      int least = 0;
      // one boundary at a time (a rolled loop: unrolled, the eight of them cost some 80 registers)
#pragma unroll 1
      for (int q = 0; q < 7; ++q) {
        const int n1 = threshold_pattern(a.thr[f][q]) - lo + 1;
        least = n1 < least ? n1 : least;
        uint32_t C;
        double S;
        hist_prefix<In>(hist, cntp, sump, keep, lo, med3i(n1, 0, nbin), C, S);
        ca = __builtin_fma(S, a.dgd[f][q], ca);
        cb4 = __mul24(static_cast<int>(C), a.dg2q[f][q]) + cb4;
      }
      if constexpr (TAIL) {
        // negative elements with a pattern above H: the short histogram's totals less its prefix
        const int n1 = threshold_pattern(a.thr[f][7]) - tlo + 1;
        least = n1 < least ? n1 : least;
        uint32_t C;
        double S;
        hist_prefix<In>(thist, tcntp, tsump, keep, tlo, med3i(n1, 0, ntbin), C, S);
        ca = __builtin_fma(tsump[ntg] - S, a.dgd[f][7], ca);
        cb4 = __mul24(static_cast<int>(tcntp[ntg] - C), a.dg2q[f][7]) + cb4;
      }
      const bool bad = least < 0;
      if (k < K) {
        const double gl = static_cast<double>(a.g_last[f]);
        const double A = ca + gl * s_total;
        const double B = 0.25 * static_cast<double>(cb4) + gl * gl * static_cast<double>(c_total);
        const double sc = static_cast<double>(s);
        const double v = (en - 2.0 * sc * A) + sc * sc * B;   // filtered error
        s_fast[f][k] = bad ? __builtin_nan("") : v;
      }
    };
    for (int u = wave; u < NF * chunks; u += NW) {
      const int f = u / chunks;                         // wave-uniform
      const int k = (u - f * chunks) * 64 + lane;
      const bool tail = (f == 0) ? TAIL_A : TAIL_B;
      if (tail) unit(std::true_type{}, f, k);
      else unit(std::false_type{}, f, k);
    }
  }
  __syncthreads();

  // ---- shortlist.  The rounding bound of the filtered error is the sorting kernel's with the depth
  // of this kernel's summation trees: a group's sum is exact (products and sum of fewer than 2^27
  // units of one ulp), a group prefix adds at most GPMAX of them in a thread, 6 levels of the wave
  // scan and the waves before, and a look-up adds two exact products: fewer than D = 16 roundings,
  // each of at most u sum|x|, whatever the row's length.
  for (int f = wave; f < NF; f += NW) {
    double m = __builtin_inf();
    int km = 0;
    float smax = 0.0f;
    for (int k = lane; k < K; k += 64) {
      const double v = s_fast[f][k];
      if (v < m) { m = v; km = k; }
      smax = __builtin_fmaxf(smax, s_scale[f][k]);
    }
    wave_argmin_dpp(m, km);
    smax = wave_max(smax);
    const double sm = static_cast<double>(smax), gm = static_cast<double>(a.g_absmax[f]);
    const double nd = static_cast<double>(n);
    const double mag = en + 2.0 * sm * gm * l1 + sm * sm * gm * gm * nd;
    const double thr = m + 0x1p-33 * mag;   // twice the margin: both values carry the error
    int cnt = 0;
    for (int k0 = 0; k0 < K; k0 += 64) {
      const int k = k0 + lane;
      cnt += __builtin_popcountll(__ballot(k < K && !(s_fast[f][k < K ? k : 0] > thr)));
    }
    static_assert(GPMAX + 6 + NW + 2 <= 16, "depth of the prefix sums");
    const double beta = 0x1p-53 * (40.0 * 16 * 2.0 * sm * l1 + (E + 32) * en + 8.0 * sm * sm * gm * gm * nd);
    const bool direct = cnt == 1 && beta <= 0x1p-34 * m;   // false for a zero or non-finite error
    if (lane == 0) { s_thr[f] = thr; s_direct[f] = direct ? km : -1; }
  }
  if (tid == 0) s_nlist = 0;
  __syncthreads();
#pragma unroll
  for (int f = 0; f < NF; ++f)
    if (s_direct[f] < 0)   // uniform
      for (int k = tid; k < K; k += THREADS)
        if (!(s_fast[f][k] > s_thr[f])) s_list[atomicAdd(&s_nlist, 1)] = static_cast<uint8_t>(f * MOFQ_MAX_CLIP + k);   // any order
  __syncthreads();
  const int n_list = s_nlist;

  // ---- exact fp64 re-score of the shortlist, element by element ------------------------------
  uint32_t carry = 0;
  for (int e = 0; e < n_list; ++e) {
    const int fk = s_list[e];
    const int f = __builtin_amdgcn_readfirstlane(fk / MOFQ_MAX_CLIP);
    const int k = __builtin_amdgcn_readfirstlane(fk % MOFQ_MAX_CLIP);
    const float s = s_scale[f][k], inv = 1.0f / s;
    const double sd = static_cast<double>(s);
    double acc = 0.0;
    // the row is read again (it left the registers after the counting; this pass is rare)
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const int64_t c0 = (static_cast<int64_t>(j) * THREADS + tid) * 8;
      u32x4 raw = {0u, 0u, 0u, 0u};   // padding is zero and scores zero
      if (c0 < a.cols) raw = *reinterpret_cast<const u32x4*>(src + c0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x0 = bits_to_float<In>(raw[i] & 0xFFFFu);
        const float x1 = bits_to_float<In>(raw[i] >> 16);
        if (f == 0) rescore2<FA>(acc, x0, x1, inv, sd, carry);
        else rescore2<FBX>(acc, x0, x1, inv, sd, carry);
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

  if (tid < NF) {
    const int f = tid;
    double best = __builtin_inf();
    int bk = s_direct[f];
    if (bk >= 0) best = s_fast[f][bk];
    for (int e = 0; e < n_list; ++e) {   // smallest error, then smallest index: the first smallest
      const int fk = s_list[e];
      if (fk / MOFQ_MAX_CLIP != f) continue;
      const int k = fk % MOFQ_MAX_CLIP;
      if (s_val[e] < best || (s_val[e] == best && k < bk)) { best = s_val[e]; bk = k; }
    }
    if (bk < 0) { bk = 0; best = __builtin_nan(""); }   // only on non-finite input
    T.rec.scale[f][row] = s_scale[f][bk];
    T.rec.clip[f][row] = bk;
    T.rec.err[f][row] = best;
    if (f == 0 && T.rec.energy) T.rec.energy[row] = en;
  }
}

// ---- host: rounding thresholds of the level boundaries ---------------------------------------

// Level magnitudes of a 4-bit format in ascending order, and for each boundary b the largest
// fp32 t = |x| / s that still lands on magnitude m_b or below.  Rounding is to nearest with ties
// to the even code, which is symmetric in the sign.
void fill_levels(int fmt, SortedArgs& a, int slot) {
  double m[9];
  bool up_is_even[8];   // at the midpoint between m[b] and m[b+1], does the tie go to m[b+1]?
  const bool int4 = fmt == MOFQ_INT4;
  if (int4) {
    for (int q = 0; q <= 8; ++q) m[q] = q;   // 8 only on the negative side
  } else {  // E2M1: magnitudes by code 0..7
    const double mag[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};
    for (int c = 0; c < 8; ++c) m[c] = mag[c];
    m[8] = mag[7];
  }
  for (int b = 0; b < 8; ++b) up_is_even[b] = ((b + 1) % 2 == 0);   // INT4: the integer b + 1; E2M1: the code b + 1
  a.g_last[slot] = static_cast<float>(m[7]);
  a.g_absmax[slot] = static_cast<float>(m[8]);
  for (int b = 0; b < 8; ++b) { a.thr[slot][b] = -INFINITY; a.dgd[slot][b] = 0.0; a.dg2q[slot][b] = 0; }
  for (int b = 0; b < 7; ++b) {
    const float mid = static_cast<float>(0.5 * (m[b] + m[b + 1]));   // exact in fp32
    // tie goes up  -> magnitude <= m_b needs t <  mid -> t <= the float just below mid
    // tie goes down-> magnitude <= m_b needs t <= mid
    a.thr[slot][b] = up_is_even[b] ? std::nextafterf(mid, -INFINITY) : mid;
    a.dgd[slot][b] = m[b] - m[b + 1];
    a.dg2q[slot][b] = static_cast<int32_t>(4.0 * (m[b] * m[b] - m[b + 1] * m[b + 1]));   // exact
  }
  if (int4) {
    // a negative element stays on -7 while t < 7.5 (the tie goes to the even 8); beyond, it lands on -8
    a.thr[slot][7] = std::nextafterf(7.5f, -INFINITY);
    a.dgd[slot][7] = m[8] - m[7];
    a.dg2q[slot][7] = static_cast<int32_t>(4.0 * (m[8] * m[8] - m[7] * m[7]));
  }
}

template <typename In, int FA, int FB>
int launch_shape(const SortedArgs& a, int64_t total_rows, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(total_rows));
  const int64_t chunks = a.cols / 8;
#define MOFQ_SORTED(THREADS, CH)                                                          \
  if (chunks <= static_cast<int64_t>(THREADS) * (CH)) {                                    \
    hipLaunchKernelGGL((sweep_sorted_kernel<In, FA, FB, THREADS, CH>), grid, dim3(THREADS), 0, st, a); \
    return hip_status(hipGetLastError());                                                  \
  }
  MOFQ_SORTED(256, 1)   //  2048 columns
  MOFQ_SORTED(256, 2)   //  4096
  MOFQ_SORTED(256, 4)   //  8192
  MOFQ_SORTED(256, 6)   // 12288
  MOFQ_SORTED(1024, 3)  // 24576
#undef MOFQ_SORTED
  return MOFQ_ERR_UNSUPPORTED;
}

// The histogram kernel: dynamic LDS for [sum prefixes | counters | count prefixes (16 bits)] of both
// histograms; the shortlist's re-scored values lie over its start later.
template <typename In, int FA, int FB>
int launch_hist_shape(const SortedArgs& a, int64_t total_rows, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(total_rows));
  const int64_t chunks = a.cols / 8;
  const int ng = a.nbin / 8, ntg = a.ntbin / 8;
  const size_t lds = std::max<size_t>((static_cast<size_t>((ng + 1) + (ntg + 1)) * 8 + 15) / 16 * 16 + 2 * static_cast<size_t>(a.nbin + a.ntbin) +
                                          2 * static_cast<size_t>((ng + 1) + (ntg + 1)),
                                      2 * MOFQ_MAX_CLIP * sizeof(double));   // at least the shortlist's values
#define MOFQ_HIST(CH)                                                                         \
  if (chunks <= 256 * (CH)) {                                                                  \
    hipLaunchKernelGGL((sweep_hist_kernel<In, FA, FB, CH>), grid, dim3(256), lds, st, a);       \
    return hip_status(hipGetLastError());                                                      \
  }
  MOFQ_HIST(1)   //  2048 columns
  MOFQ_HIST(2)   //  4096
  MOFQ_HIST(4)   //  8192
  MOFQ_HIST(6)   // 12288
  MOFQ_HIST(12)  // 24576
#undef MOFQ_HIST
  return MOFQ_ERR_UNSUPPORTED;
}

template <typename In>
int launch_fmt(const SweepParams& p, const SortedArgs& a, int64_t total_rows, hipStream_t st) {
  const int fa = p.fmt[0], fb = p.n_fmt == 2 ? p.fmt[1] : -1;
  const bool hist = a.nbin > 0;
  if (fa == MOFQ_INT4 && fb == MOFQ_FP4_E2M1)
    return hist ? launch_hist_shape<In, MOFQ_INT4, MOFQ_FP4_E2M1>(a, total_rows, st) : launch_shape<In, MOFQ_INT4, MOFQ_FP4_E2M1>(a, total_rows, st);
  if (fa == MOFQ_INT4 && fb == -1)
    return hist ? launch_hist_shape<In, MOFQ_INT4, -1>(a, total_rows, st) : launch_shape<In, MOFQ_INT4, -1>(a, total_rows, st);
  if (fa == MOFQ_FP4_E2M1 && fb == -1)
    return hist ? launch_hist_shape<In, MOFQ_FP4_E2M1, -1>(a, total_rows, st) : launch_shape<In, MOFQ_FP4_E2M1, -1>(a, total_rows, st);
  return MOFQ_ERR_UNSUPPORTED;
}

// How many bit patterns lie between a threshold t = c * amax and amax at most: a pattern is
// (exponent, mantissa) read as an integer, i.e. PPB * (log2 of the value + a term in [0, 0.0861))
// up to a constant, so two values a factor 1 / c apart are at most PPB * (log2(1 / c) + 0.0861) + 1
// patterns apart (fewer among subnormals).  The scale's own roundings move a threshold by less than
// a pattern; the kernel rounds the first counter's pattern up to a multiple of 8.
int hist_bins(double ratio_amax_over_threshold, int ppb) {
  const double lg = std::log2(ratio_amax_over_threshold);
  const double bins = ppb * ((lg > 0.0 ? lg : 0.0) + 0.09) + 24.0;
  if (!(bins < 1.0e6)) return 1 << 20;
  return (static_cast<int>(std::ceil(bins)) + 7) / 8 * 8;
}

// Sizes of the histograms for this configuration, or 0 where they would not fit (then the
// sorting kernel runs).  They depend on the formats, the clip ratios and the dtype only.
void hist_sizes(const SweepParams& p, SortedArgs& a) {
  a.nbin = 0;
  a.ntbin = 0;
  float r_min = INFINITY;
  for (int k = 0; k < p.n_clip; ++k) {
    if (!(p.clip[k] > 0.0f) || !std::isfinite(p.clip[k])) return;
    r_min = std::fmin(r_min, p.clip[k]);
  }
  const int ppb = p.dtype == MOFQ_F16 ? 1024 : 128;
  int nbin = 16, ntbin = 0;
  for (int f = 0; f < p.n_fmt; ++f) {
    const double qmax = p.fmt[f] == MOFQ_INT4 ? 7.0 : 6.0;
    nbin = std::max(nbin, hist_bins(qmax / (static_cast<double>(a.thr[f][0]) * r_min), ppb));
    if (p.fmt[f] == MOFQ_INT4) ntbin = std::max(16, hist_bins(qmax / (static_cast<double>(a.thr[f][7]) * r_min), ppb));
  }
  if (nbin > kHistMaxBins || ntbin > kHistMaxTailBins) return;
  a.nbin = nbin;
  a.ntbin = ntbin;
}

}  // namespace

// Returns MOFQ_ERR_UNSUPPORTED when the configuration is outside this kernel's domain
// (the caller then uses the direct kernel) or the tensors do not share row length, dtype and
// configuration; nothing has been enqueued in that case.
int launch_sweep_sorted_group(const SweepParams* ps, int n, hipStream_t st) {
  if (!ps || n < 1 || n > kSweepGroupMax) return MOFQ_ERR_UNSUPPORTED;
  const SweepParams& p = ps[0];
  if (p.gran != MOFQ_PER_CHANNEL) return MOFQ_ERR_UNSUPPORTED;
  if (p.dtype != MOFQ_F16 && p.dtype != MOFQ_BF16) return MOFQ_ERR_UNSUPPORTED;
  if (p.n_clip < 8 || p.cols < 1024 || p.cols > 24576) return MOFQ_ERR_UNSUPPORTED;
  for (int f = 0; f < p.n_fmt; ++f)
    if (p.fmt[f] != MOFQ_INT4 && p.fmt[f] != MOFQ_FP4_E2M1) return MOFQ_ERR_UNSUPPORTED;
  int64_t total_rows = 0;
  for (int i = 0; i < n; ++i) {
    if (ps[i].rows < 1) return MOFQ_ERR_UNSUPPORTED;
    total_rows += ps[i].rows;
  }
  if (total_rows >= (int64_t{1} << 31)) return MOFQ_ERR_UNSUPPORTED;
  for (int i = 1; i < n; ++i) {
    const SweepParams& q = ps[i];
    if (q.gran != p.gran || q.dtype != p.dtype || q.cols != p.cols ||
        q.scale_f16 != p.scale_f16 || q.n_clip != p.n_clip || q.n_fmt != p.n_fmt)
      return MOFQ_ERR_UNSUPPORTED;
    for (int f = 0; f < p.n_fmt; ++f)
      if (q.fmt[f] != p.fmt[f]) return MOFQ_ERR_UNSUPPORTED;
    for (int k = 0; k < p.n_clip; ++k)
      if (q.clip[k] != p.clip[k]) return MOFQ_ERR_UNSUPPORTED;
  }
  SortedArgs a{};
  uint32_t row0 = 0;
  for (int i = 0; i < kSweepGroupMax; ++i) {
    a.row0[i] = 0xFFFFFFFFu;
    if (i >= n) continue;
    a.t[i].w = ps[i].w;
    a.t[i].ld = ps[i].ld;
    a.t[i].rec = ps[i].rec;
    a.row0[i] = row0;
    row0 += static_cast<uint32_t>(ps[i].rows);
  }
  a.cols = p.cols;
  a.scale_f16 = p.scale_f16;
  a.n_clip = p.n_clip;
  for (int k = 0; k < p.n_clip; ++k) a.clip[k] = p.clip[k];
  for (int f = 0; f < p.n_fmt; ++f) fill_levels(p.fmt[f], a, f);
  hist_sizes(p, a);
  return p.dtype == MOFQ_F16 ? launch_fmt<F16>(p, a, total_rows, st) : launch_fmt<BF16>(p, a, total_rows, st);
}

int launch_sweep_sorted(const SweepParams& p, hipStream_t st) { return launch_sweep_sorted_group(&p, 1, st); }

}  // namespace mofq
