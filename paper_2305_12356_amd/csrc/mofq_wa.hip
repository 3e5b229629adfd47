// Layer-output error of a weight-activation quantized linear layer (Section 3.2,
// layer analysis: A_out = W * A_in with both inputs quantized):
//
//     E_f = sum_{t,o} ( Y[t,o] - sx_f * sw_f[o] * (Qx_f Qw_f^T)[t,o] )^2 ,  P = sum Y^2 ,
//     Y = X W^T .
//
// One kernel computes, per 256x128 output tile, the reference product on the bf16
// matrix cores, then up to two quantized products (for W8A8: the INT8 code product on the
// int8 matrix cores and the FP8-E4M3 code product), one after the other: each product is a K loop of its own over its own
// operand arrays, the reference accumulators stay in registers for the whole kernel and
// the quantized accumulators are reduced against them (squared differences in fp64) as
// soon as their loop ends.  Y is never written to memory.
//
// Why the products run in sequence and not side by side: the loop is bound by the
// texture path (one 128-byte line every ~2.2 clocks per compute unit, whatever part of
// the line is used), by LDS bandwidth and by how many bytes can be in flight from L2
// into LDS.  One product at a time lets a stage hold whole 128-byte lines of every
// operand row (48 KB, three stages resident) and keeps a wave at two accumulator sets
// (128 registers for its 64x64 share), so that eight waves, two per SIMD, fit: while
// one waits at the stage barrier or for its fragments the other keeps the matrix core
// busy.  The 256x128 workgroup tile needs 25 % fewer operand bytes per flop than
// 128x128.
//
// Exactness: bf16 x bf16 products are exact in fp32 and are accumulated in fp32;
// int8 products are accumulated exactly in int32 (|sum| <= 32768*127*127 < 2^31).
// A quantized product is one of three kinds:
//   WA_INT8      : int8 codes on the int8 matrix cores (exact);
//   WA_GRID_BF16 : grid values stored as bf16 (exact for 4-bit and 8-bit grids) on the
//                  bf16 matrix cores, products exact, fp32 accumulation -- the E4M3
//                  product that meets the 1e-5 tolerance on the error sum, and the
//                  4-bit products of the weight-only layer-output metric, where the
//                  "quantized" input is the 16-bit input itself (scale 1);
//   WA_FP8       : e4m3 codes on the fp8 matrix cores (the low-bit matmul units the WA
//                  case of Algorithm 1 targets).  Measured on the part with single
//                  instructions: the 8 products of each group of 8 consecutive k are
//                  aligned to the group's largest exponent sum (operand exponents added,
//                  whatever the mantissas) and bits more than 13 places below it are
//                  dropped towards zero; the group sums and the accumulator are then added
//                  like fp32 numbers.  On tensors with outlier channels that shifts the
//                  error sum by 1e-6 .. 3e-5 relative, more where a layer's largest outliers
//                  stretch its scales further, plus a random part that falls with the
//                  number of outputs (a few 1e-5 at some ten thousand outputs).  A caller can
//                  keep the outlier columns out of this product (zeros in the X operand) and
//                  hand their grid values over as a second part (QProd::xs / ws): one K step
//                  on the bf16 matrix cores into the same accumulators, which brings the sum
//                  to within 4e-7 at full size.
#include <type_traits>

#include "mofq_device.h"
#include "mofq_internal.h"

namespace mofq {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int SIDE_K = kWaSideCols;             // K extent of a product's optional second part: one 16-bit stage
constexpr int TM = 256, TN = 128;               // workgroup tile; 8 waves (two per SIMD), 64 x 64 each
constexpr int WM = 64, WN = 64;                 // wave tile: 2 x 2 matrix-core tiles of 32 x 32
constexpr int NW = (TM / WM) * (TN / WN);       // waves per workgroup
constexpr int TI = WM / 32, TJ = WN / 32;

struct QProd {
  const void* x; const void* w;                 // dense [M][K], [N][K] in the product's operand type
  const float* sx; const float* sw;             // scales: sx one value or null (= 1); sw one value or [N]
  double* part;                                 // [blocks]
  const void* xs; const void* ws;               // optional second part: bf16 grid values, dense [M][SIDE_K], [N][SIDE_K]
};
struct GemmArgs {
  const uint16_t* x; int64_t ldx;               // bf16 [M][K]
  const uint16_t* w; int64_t ldw;               // bf16 [N][K]
  QProd q[2];
  int32_t w_per_channel;
  int32_t M, N, K;
  int32_t tiles_m, tiles_n;
  double* part_p;                               // [blocks]
};

// ---- LDS stage ----------------------------------------------------------------------
// A stage holds one K slab of both operand tiles: 256 rows of X then 128 rows of W, each
// row ROW_B = 128 bytes (64 sixteen-bit or 128 eight-bit elements, one cache line), i.e.
// 8 chunks of 16 bytes, no padding.  Stages are filled by global_load_lds (each lane of a wave
// instruction deposits 16 bytes at consecutive LDS addresses), so the layout is chosen
// through WHICH global chunk a lane fetches: chunk slot p of row R holds logical chunk
// p ^ swz(R).  A 128-bit LDS read is served 16 lanes (256 bytes, all 64 banks) per
// clock; the 16 lanes of one pass read the same logical chunk of 16 consecutive rows,
// which by themselves cover 2 distinct 128-byte offsets, so the rotation advances once
// every 2 rows.
constexpr int ROW_B = 128;
constexpr int CH = ROW_B / 16;                  // chunks per row
constexpr int STAGE_ROWS = TM + TN;
constexpr int STAGE = STAGE_ROWS * ROW_B;       // 48 KB
constexpr int NST = 3;                          // stages resident
constexpr int AHEAD = NST - 1;                  // stage kt + AHEAD is issued during step kt
constexpr int DEP = STAGE / 1024 / NW;          // deposits per wave per stage (6)
MOFQ_DEV constexpr int swz(int row) { return (row >> 1) & (CH - 1); }

// One wave instruction: lane l fetches 16 bytes at its own global address and deposits
// them at LDS address lds_base + 16*l.  Written as inline assembly so that the compiler
// does not serialise later LDS reads of OTHER buffers behind the deposit; completion is
// tracked by hand with s_waitcnt vmcnt (deposits of a wave retire in order).
MOFQ_DEV void lds_deposit(const char* gsrc, const unsigned char* lds_dst) {
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) const unsigned char*)lds_dst));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(gsrc)
               : "memory");   // m0 is not otherwise used by these kernels
}

// s_waitcnt with only the vector-memory counter constrained (6 bits, split field).
template <int N> MOFQ_DEV void wait_deposits_but() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

enum : int { K_REF = 100, K_GRID = WA_GRID_BF16, K_I8 = WA_INT8, K_F8 = WA_FP8 };   // K_REF: the 16-bit inputs themselves

template <int KIND1, int KIND2>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void wa_gemm_kernel(const GemmArgs a) {
  __shared__ __attribute__((aligned(1024))) unsigned char s_buf[NST * STAGE];
  __shared__ double s_red[3][NW];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;      // 4 x 2 waves
  const int r = lane & 31, g = lane >> 5;

  // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs (8 of them, each
  // with its own L2), so ids are first regrouped so that one XCD works on a contiguous
  // range of tiles, and a range is walked in bands of 4 tile rows: the 32 workgroups
  // resident on an XCD then share 4 X tiles and 8 W tiles.
  int t = blockIdx.x;
  {
    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = total / 8;
    if (t < per_xcd * 8) t = (t & 7) * per_xcd + (t >> 3);
    constexpr int BAND = 4;
    const int band = t / (BAND * a.tiles_n);
    const int first_m = band * BAND;
    const int rows_in_band = (a.tiles_m - first_m) < BAND ? (a.tiles_m - first_m) : BAND;
    const int in_band = t - band * BAND * a.tiles_n;
    const int bm_ = first_m + in_band % rows_in_band;
    const int bn_ = in_band / rows_in_band;
    t = bm_ * a.tiles_n + bn_;
  }
  const int bm = t / a.tiles_n, bn = t - bm * a.tiles_n;
  const int m0 = bm * TM, n0 = bn * TN;

  // LDS byte offsets of this lane's fragment rows inside a stage, and of the chunks it
  // reads: lane (r, g) supplies row r of a 32-row operand tile and the g-th half of the
  // instruction's K range, for A and B alike.
  const int sw = swz(r);                                   // same for all of the lane's rows (multiples of 32 apart)
  const int row_a = (wm * WM + r) * ROW_B;                 // + i * 32 * ROW_B
  const int row_b = (TM + wn * WN + r) * ROW_B;            // + j * 32 * ROW_B
  int ch_k[CH / 2], ch_f[CH / 2];
#pragma unroll
  for (int q = 0; q < CH / 2; ++q) {
    ch_k[q] = ((2 * q + g) ^ sw) * 16;                       // K slice q of a stage, 16 bytes per lane
    ch_f[q] = ((4 * (q >> 1) + 2 * g + (q & 1)) ^ sw) * 16;  // fp8 instruction q/2: 32 bytes per lane, half q%2
  }

  f32x16 acc_r[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc_r[i][j][e] = 0.0f;

  // ---- one product: K loop over its own operand arrays ---------------------------------
  // KIND selects arrays, element size and matrix instruction; acc is f32x16 or i32x16.
  auto product = [&](auto kind_c, auto& acc, const void* xq, const void* wq, const int kdim) {
    constexpr int KIND = decltype(kind_c)::value;
    constexpr int EB = (KIND == K_REF || KIND == K_GRID) ? 2 : 1;   // bytes per element
    constexpr int TK = ROW_B / EB;                                  // K elements per stage
    constexpr int NG = (KIND == K_F8) ? CH / 4 : CH / 2;            // matrix groups per stage (TI*TJ instructions each)
    constexpr int NF = (KIND == K_F8) ? 2 : 1;                      // 16-byte chunks per fragment
    const char* xb; const char* wb; int64_t xrow, wrow;
    if constexpr (KIND == K_REF) { xb = reinterpret_cast<const char*>(a.x); wb = reinterpret_cast<const char*>(a.w); xrow = a.ldx * 2; wrow = a.ldw * 2; }
    else { xb = static_cast<const char*>(xq); wb = static_cast<const char*>(wq); xrow = wrow = static_cast<int64_t>(kdim) * EB; }

    // This lane's global source of each of its wave's deposits at k = 0 (deposit i of a
    // stage covers chunk slots 64 i .. 64 i + 63 and is issued by wave i % NW).
    const char* src[DEP];
#pragma unroll
    for (int d = 0; d < DEP; ++d) {
      const int c = (wave + NW * d) * 64 + lane;
      const int row = c / CH, kc = (c % CH) ^ swz(row);
      if (row < TM) {
        int gr = m0 + row;
        gr = gr < a.M ? gr : a.M - 1;          // rows past the edge repeat the last one (masked later)
        src[d] = xb + static_cast<int64_t>(gr) * xrow + kc * 16;
      } else {
        int gr = n0 + row - TM;
        gr = gr < a.N ? gr : a.N - 1;
        src[d] = wb + static_cast<int64_t>(gr) * wrow + kc * 16;
      }
    }
    // K is a multiple of 64 elements, so the last stage of an 8-bit product may hold only
    // half a row (64 bytes).  Its deposits then fetch the valid half twice (addresses stay
    // inside the row) and the matrix groups of the missing half are skipped.
    const int KT = (kdim + TK - 1) / TK;
    const bool half_tail = (EB == 1) && (kdim % TK) != 0;   // 16-bit stages hold 64 elements: never
    auto issue = [&](int kt, int lo, int hi) {   // deposits [lo, hi) of stage kt
      unsigned char* st = s_buf + (kt % NST) * STAGE;
      const int64_t kb = static_cast<int64_t>(kt) * ROW_B;
      const bool tail = half_tail && kt == KT - 1;
#pragma unroll
      for (int d = 0; d < DEP; ++d)
        if (d >= lo && d < hi) {
          const char* g_src = src[d] + kb;
          if (tail) {
            const int c = (wave + NW * d) * 64 + lane;
            if (((c % CH) ^ swz(c / CH)) >= CH / 2) g_src -= ROW_B / 2;
          }
          lds_deposit(g_src, st + (wave + NW * d) * 1024);
        }
    };
    // Fragments of group gi of a stage: f[0 .. TI*NF) = A tiles, f[TI*NF ..) = B tiles.
    auto load_group = [&](const unsigned char* st, int gi, i32x4 (&f)[(TI + TJ) * NF]) {
#pragma unroll
      for (int h = 0; h < NF; ++h) {
        const int ch = (KIND == K_F8) ? ch_f[2 * gi + h] : ch_k[gi];
#pragma unroll
        for (int i = 0; i < TI; ++i) f[i * NF + h] = *reinterpret_cast<const i32x4*>(st + row_a + i * 32 * ROW_B + ch);
#pragma unroll
        for (int j = 0; j < TJ; ++j) f[(TI + j) * NF + h] = *reinterpret_cast<const i32x4*>(st + row_b + j * 32 * ROW_B + ch);
      }
    };
    // The matrix instructions of one group, with the deposits [lo, hi) of stage kt_dep
    // spread between them: a wave issues in order, so a burst of deposits (each occupies
    // the texture path for ~18 clocks, and all waves share it) would hold back the
    // matrix instructions behind it while the matrix pipe runs dry.
    auto run_group = [&](const i32x4 (&f)[(TI + TJ) * NF], bool more, int kt_dep, int lo, int hi) {
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
          {
            const int m = i * TJ + j, n = hi - lo;
            __builtin_amdgcn_sched_barrier(0);
            if (more) issue(kt_dep, lo + m * n / (TI * TJ), lo + (m + 1) * n / (TI * TJ));
            __builtin_amdgcn_sched_barrier(0);
          }
          if constexpr (KIND == K_REF || KIND == K_GRID) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f[i]), __builtin_bit_cast(bf16x8, f[TI + j]), acc[i][j], 0, 0, 0);
          } else if constexpr (KIND == K_I8) {
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f[i], f[TI + j], acc[i][j], 0, 0, 0);
          } else {
            i32x8 fa, fb;
#pragma unroll
            for (int e = 0; e < 4; ++e) { fa[e] = f[i * 2][e]; fa[4 + e] = f[i * 2 + 1][e]; fb[e] = f[(TI + j) * 2][e]; fb[4 + e] = f[(TI + j) * 2 + 1][e]; }
            // format selectors 0 = E4M3 for both operands; block scales 2^0 (exponent byte 127)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa, fb, acc[i][j], 0, 0, 0, 127, 0, 127);
          }
        }
    };
    // Wait until this wave's deposits of stage kt have landed; those of stage kt+1 (if
    // there is one) may stay in flight.
    auto wait_stage = [&](int kt) {
      if (kt + 1 < KT) wait_deposits_but<DEP>();
      else wait_deposits_but<0>();
    };

    // Prologue: AHEAD stages on their way.
#pragma unroll
    for (int s = 0; s < AHEAD; ++s)
      if (s < KT) issue(s, 0, DEP);

    // One K step: the barrier makes stage kt visible to everyone and tells everyone that
    // stage kt-1 is no longer read, which is the buffer the deposits of stage kt+AHEAD go
    // to.  Inside the step the fragments of group g+1 are requested before the matrix
    // instructions of group g are issued, and the deposits are spread over the groups so
    // that the texture path works while the matrix cores do.
    auto step = [&](int kt, auto groups_c) {
      constexpr int GROUPS = decltype(groups_c)::value;
      wait_stage(kt);
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");     // LDS reads below must not move above the barrier
      const unsigned char* st = s_buf + (kt % NST) * STAGE;
      const bool more = kt + AHEAD < KT;
      i32x4 f[2][(TI + TJ) * NF];
      load_group(st, 0, f[0]);
#pragma unroll
      for (int gi = 0; gi < GROUPS; ++gi) {
        if (gi + 1 < GROUPS) load_group(st, gi + 1, f[(gi + 1) & 1]);
        run_group(f[gi & 1], more, kt + AHEAD, gi * DEP / GROUPS, (gi + 1) * DEP / GROUPS);
      }
    };
    const int KT_full = half_tail ? KT - 1 : KT;
    for (int kt = 0; kt < KT_full; ++kt) step(kt, std::integral_constant<int, NG>{});
    if constexpr (EB == 1)
      if (half_tail) step(KT - 1, std::integral_constant<int, NG / 2>{});
    // All deposits of this product have landed (the last wait allowed none in flight);
    // the next product's prologue overwrites buffers only after everyone is here.
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // ---- squared differences in fp64.  Accumulator value e of a lane in one 32x32 tile is
  // output (row 8*(e/4) + 4*g + e%4, column lane%32) of that tile; rows and columns past
  // the matrix edge hold repeats of the last row and are skipped.  The first reduction
  // also sums Y^2.
  double p = 0.0;
  auto sq_diff = [&](auto with_p_c, const auto& acc_q, const float* sx, const float* sw_) {
    constexpr bool WITH_P = decltype(with_p_c)::value;
    __builtin_amdgcn_sched_barrier(0);
    const double sxd = sx ? static_cast<double>(*sx) : 1.0;
    double e_q = 0.0;
    // rows of this lane's accumulators that exist: 32 i + 8 (e/4) + e%4 < row_lim.  Opaque,
    // so that each reduction computes its own masks instead of keeping 128 of them live.
    int row_lim = a.M - (m0 + wm * WM + 4 * g);
    asm volatile("" : "+v"(row_lim));
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
      const int n = n0 + wn * WN + j * 32 + r;
      const bool col_ok = n < a.N;
      const int ns = (a.w_per_channel && col_ok) ? n : 0;
      const double cq = sxd * static_cast<double>(sw_[ns]);
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const bool ok = col_ok && (i * 32 + 8 * (e / 4) + (e % 4)) < row_lim;
          // Opaque copy, ordered after the previous element's sum.  Without it the fp64
          // image of all 128 reference values is kept (spilled) across the next product's
          // K loop for reuse in its reduction, and the conversions of all elements are
          // hoisted ahead of the two summation chains, which spills as well: every
          // register is in use here.
          float yf = acc_r[i][j][e];
          asm volatile("" : "+v"(yf) : "v"(e_q));
          const double y = ok ? static_cast<double>(yf) : 0.0;
          const double q = ok ? static_cast<double>(acc_q[i][j][e]) : 0.0;
          const double d = __builtin_fma(-cq, q, y);
          e_q = __builtin_fma(d, d, e_q);
          if constexpr (WITH_P) p = __builtin_fma(y, y, p);
        }
    }
    // Pin the sums here: otherwise the Y^2 chain is sunk to the end of the kernel and
    // its 128 fp64 inputs are spilled across the next product.
    asm volatile("" : "+v"(e_q), "+v"(p));
    __builtin_amdgcn_sched_barrier(0);   // and keep the next product's set-up out of this reduction
    return wave_sum(e_q);
  };

  product(std::integral_constant<int, K_REF>{}, acc_r, nullptr, nullptr, a.K);
  double e_q[2] = {0.0, 0.0};
  auto quantized = [&](auto kind_c, auto slot_c) {
    constexpr int KIND = decltype(kind_c)::value;
    constexpr int SLOT = decltype(slot_c)::value;
    if constexpr (KIND != WA_NONE) {
      using acc_t = std::conditional_t<KIND == K_I8, i32x16, f32x16>;
      acc_t acc_q[TI][TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc_q[i][j][e] = 0;
      product(kind_c, acc_q, a.q[SLOT].x, a.q[SLOT].w, a.K);
      // The columns split off from an fp8-unit product: one K step from their grid values on
      // the bf16 matrix cores into the same accumulators (both accumulate in fp32).
      if constexpr (KIND == K_F8)
        if (a.q[SLOT].xs) product(std::integral_constant<int, K_GRID>{}, acc_q, a.q[SLOT].xs, a.q[SLOT].ws, SIDE_K);
      // the first reduction also sums Y^2
      e_q[SLOT] = sq_diff(std::integral_constant<bool, SLOT == 0>{}, acc_q, a.q[SLOT].sx, a.q[SLOT].sw);
    }
  };
  quantized(std::integral_constant<int, KIND1>{}, std::integral_constant<int, 0>{});
  quantized(std::integral_constant<int, KIND2>{}, std::integral_constant<int, 1>{});
  p = wave_sum(p);
  if (lane == 0) { s_red[0][wave] = e_q[0]; s_red[1][wave] = e_q[1]; s_red[2][wave] = p; }
  __syncthreads();
  if (tid == 0) {
    const int out = bm * a.tiles_n + bn;
    double t[3] = {0.0, 0.0, 0.0};
    for (int q = 0; q < 3; ++q)
      for (int w = 0; w < NW; ++w) t[q] += s_red[q][w];   // fixed order
    if (a.q[0].part) a.q[0].part[out] = t[0];
    if (a.q[1].part) a.q[1].part[out] = t[1];
    a.part_p[out] = t[2];
  }
}

}  // namespace

int wa_gemm_blocks(int64_t M, int64_t N) {
  return static_cast<int>(((M + TM - 1) / TM) * ((N + TN - 1) / TN));
}

int launch_wa_gemm(const WaGemmParams& p, hipStream_t st) {
  if (p.K % 64 != 0) return MOFQ_ERR_UNSUPPORTED;
  if (p.q[0].kind == WA_NONE) return MOFQ_ERR_INVALID_ARG;   // the first slot carries the Y^2 sum
  GemmArgs a{};
  a.x = static_cast<const uint16_t*>(p.x); a.ldx = p.ldx;
  a.w = static_cast<const uint16_t*>(p.w); a.ldw = p.ldw;
  for (int i = 0; i < 2; ++i) {
    if ((p.q[i].xs != nullptr) != (p.q[i].ws != nullptr)) return MOFQ_ERR_INVALID_ARG;
    if (p.q[i].xs && p.q[i].kind != WA_FP8) return MOFQ_ERR_INVALID_ARG;
    a.q[i] = QProd{p.q[i].x, p.q[i].w, p.q[i].sx, p.q[i].sw, p.q[i].part, p.q[i].xs, p.q[i].ws};
  }
  a.w_per_channel = p.w_per_channel;
  a.M = static_cast<int32_t>(p.M); a.N = static_cast<int32_t>(p.N); a.K = static_cast<int32_t>(p.K);
  a.tiles_m = static_cast<int32_t>((p.M + TM - 1) / TM);
  a.tiles_n = static_cast<int32_t>((p.N + TN - 1) / TN);
  a.part_p = p.part_p;
  const dim3 grid(static_cast<unsigned>(wa_gemm_blocks(p.M, p.N)));
  const int k1 = p.q[0].kind, k2 = p.q[1].kind;
  bool launched = false;
#define MOFQ_WA(A, B) \
  if (k1 == (A) && k2 == (B)) { hipLaunchKernelGGL((wa_gemm_kernel<A, B>), grid, dim3(NW * 64), 0, st, a); launched = true; }
  MOFQ_WA(WA_INT8, WA_GRID_BF16) MOFQ_WA(WA_INT8, WA_FP8) MOFQ_WA(WA_INT8, WA_NONE)
  MOFQ_WA(WA_GRID_BF16, WA_NONE) MOFQ_WA(WA_FP8, WA_NONE) MOFQ_WA(WA_GRID_BF16, WA_GRID_BF16)
#undef MOFQ_WA
  if (!launched) return MOFQ_ERR_UNSUPPORTED;
  return hip_status(hipGetLastError());
}

}  // namespace mofq
