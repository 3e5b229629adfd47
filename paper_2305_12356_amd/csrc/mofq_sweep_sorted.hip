// Scale search for one output channel per workgroup without scoring every
// (element, candidate) pair: Algorithm 1's quantize_layer + compute_error with the tensor-error
// metric (Section 4.1) for per-channel weight scales (Section 3.2, Section 5) over a table of
// clip ratios, for the 4-bit pair of Section 4.2 (INT4, FP4-E2M1 of Table 1).  Two kernels share the formulation below: sweep_sorted_kernel
// (this file) sorts the row and searches it; sweep_hist_kernel (mofq_sweep_hist.hip, with its
// own description) counts the row's bit patterns instead and is the one that runs wherever the
// clip ratios let its histogram fit, which includes the usual [0.5, 1].  This file also holds
// the host side of both: level thresholds, the histogram's size, the dispatch.
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
#include "mofq_search_common.h"

namespace mofq {

namespace {

// Padded position of sorted element i (in elements): a 2-element gap after every 64.
// Additive over sums of distinct powers of two, which the search below relies on.
MOFQ_DEV constexpr int phys(int i) { return i + ((i >> 6) << 1); }


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

template <typename In>
int launch_fmt(const SweepParams& p, const SortedArgs& a, int64_t total_rows, hipStream_t st) {
  const int fa = p.fmt[0], fb = p.n_fmt == 2 ? p.fmt[1] : -1;
  const bool hist = a.nbin > 0;
  if (fa == MOFQ_INT4 && fb == MOFQ_FP4_E2M1)
    return hist ? launch_sweep_hist(p, a, total_rows, st) : launch_shape<In, MOFQ_INT4, MOFQ_FP4_E2M1>(a, total_rows, st);
  if (fa == MOFQ_INT4 && fb == -1)
    return hist ? launch_sweep_hist(p, a, total_rows, st) : launch_shape<In, MOFQ_INT4, -1>(a, total_rows, st);
  if (fa == MOFQ_FP4_E2M1 && fb == -1)
    return hist ? launch_sweep_hist(p, a, total_rows, st) : launch_shape<In, MOFQ_FP4_E2M1, -1>(a, total_rows, st);
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
