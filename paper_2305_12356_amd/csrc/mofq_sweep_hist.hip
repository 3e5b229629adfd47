// Per-channel scale search from a histogram of the magnitudes' bit patterns: Algorithm 1's
// quantize_layer + compute_error with the tensor-error metric (Section 4.1) for per-channel weight
// scales over a table of clip ratios, INT4 against FP4-E2M1 (Table 1).  The formulation, the filter
// and the shortlist are described at the top of mofq_sweep_sorted.hip, whose kernel this one replaces
// wherever its histogram fits.
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
#include "mofq_search_common.h"

namespace mofq {

namespace {

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
    // Counter b is the low (b even) or high half of word b / 2: add 1 or 65536.  Address and
    // addend are written out (a shift-add and a mask on the LDS byte address, one 24-bit
    // multiply-add): left to the compiler the increment costs twice the instructions, and this
    // loop runs once per element.
    typedef __attribute__((address_space(3))) uint32_t lds_u32;
    const uint32_t hist_at = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_u32*)hist));     // LDS byte addresses, multiples of 16
    const uint32_t thist_at = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_u32*)thist));
    auto count = [](uint32_t at, uint32_t ub) {
      uint32_t one_or_65536;
      asm("v_mad_u32_u24 %0, %1, %2, 1" : "=v"(one_or_65536) : "v"(ub & 1u), "s"(0xFFFFu));
      lds_u32* const word = (lds_u32*)static_cast<uintptr_t>(((ub << 1) + at) & ~3u);
      __hip_atomic_fetch_add(word, one_or_65536, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto lo16 = [](i16x2 v) { return static_cast<uint32_t>(__builtin_bit_cast(uint32_t, v) & 0xFFFFu); };
    auto hi16 = [](i16x2 v) { return static_cast<uint32_t>(__builtin_bit_cast(uint32_t, v) >> 16); };
#pragma unroll
    for (int j = 0; j < CH; ++j) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t w = rawv[j][i];
        const i16x2 h2 = __builtin_bit_cast(i16x2, w & 0x7FFF7FFFu);
        const i16x2 b2 = __builtin_elementwise_min(h2 - lo2, last2);
        // padding (zero) and whatever lies below every threshold has no counter
        if (b2[0] >= 0) count(hist_at, lo16(b2));   // non-negative: the 16 bits are the counter's number
        if (b2[1] >= 0) count(hist_at, hi16(b2));
        if constexpr (ANY_TAIL) {
          const i16x2 t2 = h2 - tlo2;
          // halves that are negative elements at or above the short histogram's first pattern
          const uint32_t q2 = sign_fill2(w) & ~sign_fill2(__builtin_bit_cast(uint32_t, t2));
          if (q2 != 0) {
            const i16x2 tc2 = __builtin_elementwise_min(t2, tlast2);
            if (q2 & 0xFFFFu) count(thist_at, lo16(tc2));
            if (q2 >> 16) count(thist_at, hi16(tc2));
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

}  // namespace

int launch_sweep_hist(const SweepParams& p, const SortedArgs& a, int64_t total_rows, hipStream_t st) {
  if (a.nbin <= 0 || (p.dtype != MOFQ_F16 && p.dtype != MOFQ_BF16)) return MOFQ_ERR_UNSUPPORTED;
  const int fa = p.fmt[0], fb = p.n_fmt == 2 ? p.fmt[1] : -1;
  const bool h = p.dtype == MOFQ_F16;
  if (fa == MOFQ_INT4 && fb == MOFQ_FP4_E2M1)
    return h ? launch_hist_shape<F16, MOFQ_INT4, MOFQ_FP4_E2M1>(a, total_rows, st) : launch_hist_shape<BF16, MOFQ_INT4, MOFQ_FP4_E2M1>(a, total_rows, st);
  if (fa == MOFQ_INT4 && fb == -1)
    return h ? launch_hist_shape<F16, MOFQ_INT4, -1>(a, total_rows, st) : launch_hist_shape<BF16, MOFQ_INT4, -1>(a, total_rows, st);
  if (fa == MOFQ_FP4_E2M1 && fb == -1)
    return h ? launch_hist_shape<F16, MOFQ_FP4_E2M1, -1>(a, total_rows, st) : launch_hist_shape<BF16, MOFQ_FP4_E2M1, -1>(a, total_rows, st);
  return MOFQ_ERR_UNSUPPORTED;
}

}  // namespace mofq
