// Layer-output error of a weight-activation quantized linear layer (Section 3.2,
// layer analysis: A_out = W * A_in with both inputs quantized):
//
//     E_f = sum_{t,o} ( Y[t,o] - sx_f * sw_f[o] * (Qx_f Qw_f^T)[t,o] )^2 ,  P = sum Y^2 ,
//     Y = X W^T .
//
// One kernel computes, per 128x128 output tile, the reference product on the bf16
// matrix cores, the INT8 code product on the int8 matrix cores and the FP8-E4M3
// code product, then reduces the squared differences in fp64.  Y is never written
// to memory.
//
// Exactness: bf16 x bf16 products are exact in fp32 and are accumulated in fp32;
// int8 products are accumulated exactly in int32 (|sum| <= 32768*127*127 < 2^31).
// The E4M3 code product has two modes:
//   FP8_EXACT  : the grid values (exact in bf16) go through the bf16 matrix cores,
//                products exact, fp32 accumulation -- the mode that meets the 1e-5
//                tolerance on the error sum;
//   FP8_NATIVE : the codes go through the fp8 matrix cores (the low-bit matmul units
//                the WA case of Algorithm 1 targets).  Measured on the part: inside
//                one instruction, products are aligned per group of 8 and addends
//                below 2^-13 of the group's largest product are truncated, which
//                shifts the error sum by ~1e-5..1e-4 relative on tensors with
//                outlier channels.
#include "mofq_device.h"
#include "mofq_internal.h"

namespace mofq {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int TM = 128, TN = 128;               // workgroup tile; 4 waves, 64 x 64 each

struct GemmArgs {
  const uint16_t* x; int64_t ldx;               // bf16 [M][K]
  const uint16_t* w; int64_t ldw;               // bf16 [N][K]
  const uint8_t* xi; const uint8_t* wi;         // int8 codes, dense [M][K], [N][K]
  const uint8_t* xf; const uint8_t* wf;         // e4m3 codes (FP8_NATIVE)
  const uint16_t* xg; const uint16_t* wg;       // e4m3 grid values as bf16 (FP8_EXACT)
  const float* sx_i; const float* sw_i;         // scales: sx one value; sw one value or [N]
  const float* sx_f; const float* sw_f;
  int32_t w_per_channel;
  int32_t M, N, K;
  int32_t tiles_n;
  double* part_i; double* part_f; double* part_p;   // [blocks]
};

constexpr int FP8_NONE = 0, FP8_NATIVE = 1, FP8_EXACT = 2;

// ---- LDS tiles --------------------------------------------------------------------
// A tile holds 128 rows of RB bytes (RB = 32, 64 or 128), i.e. C = RB/16 chunks of 16
// bytes per row, with no padding.  Tiles are filled by global_load_lds (each lane of a
// wave instruction deposits 16 bytes at consecutive LDS addresses), so the layout is
// chosen through WHICH global chunk a lane fetches: chunk slot p of row R holds logical
// chunk p ^ swz(R), a rotation that spreads the 16-byte column read by the matrix-core
// fragment loads over all bank groups.
// A 128-bit LDS read is served 16 lanes (256 bytes, all 64 banks) per clock; the 16
// lanes of one pass read the same logical chunk of 16 consecutive rows, which cover
// 16/C distinct 256-byte offsets by themselves, so the rotation advances once every
// 16/C rows.
MOFQ_DEV constexpr int swz(int C, int row) { return (row / (16 / C)) % C; }
MOFQ_DEV constexpr int chunk_off(int C, int row, int kc) { return (row * C + (kc ^ swz(C, row))) * 16; }

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

// Compile-time plan of one K step: which operand tiles a stage holds, which deposits one
// wave issues for it ("slots"), and the order of the matrix-core groups (4 instructions
// on one 64 x 64 wave tile each).  A tile of C chunks per row is 2*C wave deposits,
// deposit i issued by wave i % 4.
enum : int { K_REF = 0, K_GRID = 1, K_I8 = 2, K_F8 = 3 };
struct Slot { int kind, is_w, off, C, j; };
struct Group { int kind, ks; };

template <bool DO_I8, int FP8>
struct Plan {
  static constexpr int TK = (FP8 == FP8_NATIVE) ? 64 : 32;   // the fp8 instruction consumes K = 64
  static constexpr int CB = TK * 2 / 16;                     // chunks per row, 16-bit tiles
  static constexpr int CQ = TK / 16;                         // chunks per row, 8-bit tiles
  static constexpr int SZB = TM * TK * 2, SZQ = TM * TK;     // bytes per tile
  static constexpr bool GRID = FP8 == FP8_EXACT, F8 = FP8 == FP8_NATIVE;
  static constexpr int O_XB = 0, O_WB = O_XB + SZB;
  static constexpr int O_XG = O_WB + SZB, O_WG = O_XG + (GRID ? SZB : 0);
  static constexpr int O_XI = O_WG + (GRID ? SZB : 0), O_WI = O_XI + (DO_I8 ? SZQ : 0);
  static constexpr int O_XF = O_WI + (DO_I8 ? SZQ : 0), O_WF = O_XF + (F8 ? SZQ : 0);
  static constexpr int STAGE = O_WF + (F8 ? SZQ : 0);
  // Stages in flight: a deposit takes a few thousand clocks to arrive while one stage of
  // matrix work is ~700, so loads are issued two stages ahead where LDS allows it.
  static constexpr int NST = (3 * STAGE <= 150 * 1024) ? 3 : 2;
  static constexpr int PWB = CB / 2, PWQ = CQ / 2;           // deposits per wave per tile
  static constexpr int LPS = 2 * PWB * (GRID ? 2 : 1) + 2 * PWQ * ((DO_I8 ? 1 : 0) + (F8 ? 1 : 0));
  static constexpr int off_of(int kind, int is_w) {
    return kind == K_REF ? (is_w ? O_WB : O_XB) : kind == K_GRID ? (is_w ? O_WG : O_XG)
         : kind == K_I8 ? (is_w ? O_WI : O_XI) : (is_w ? O_WF : O_XF);
  }
  static constexpr Slot slot(int s) {
    const int kinds[4] = {K_REF, K_GRID, K_I8, K_F8};
    const bool on[4] = {true, GRID, DO_I8, F8};
    for (int q = 0; q < 4; ++q) {
      if (!on[q]) continue;
      const int pw = (q < 2) ? PWB : PWQ;
      for (int is_w = 0; is_w < 2; ++is_w) {
        if (s < pw) return Slot{kinds[q], is_w, off_of(kinds[q], is_w), (q < 2) ? CB : CQ, s};
        s -= pw;
      }
    }
    return Slot{0, 0, 0, CB, 0};
  }
  // Matrix-core groups of one stage, ordered so that the three products alternate.
  static constexpr int NREF = TK / 16, NI8 = DO_I8 ? TK / 32 : 0;
  static constexpr int NG = NREF * (GRID ? 2 : 1) + NI8 + (F8 ? 1 : 0);
  static constexpr Group group(int g) {
    if (GRID) {                       // ref0 grid0 ref1 grid1 [i8]
      if (g < 2 * NREF) return Group{(g & 1) ? K_GRID : K_REF, g >> 1};
      return Group{K_I8, g - 2 * NREF};
    }
    if (F8) {                         // TK = 64: ref0 ref1 [i8_0] ref2 ref3 [i8_1] f8
      if (g == NG - 1) return Group{K_F8, 0};
      if (!DO_I8) return Group{K_REF, g};
      if (g % 3 == 2) return Group{K_I8, g / 3};
      return Group{K_REF, (g / 3) * 2 + g % 3};
    }
    if (g < NREF) return Group{K_REF, g};   // ref0 ref1 i8
    return Group{K_I8, g - NREF};
  }
};

template <bool DO_I8, int FP8>
__global__ __launch_bounds__(256) void wa_gemm_kernel(const GemmArgs a) {
  using P = Plan<DO_I8, FP8>;
  constexpr bool DO_F8 = FP8 != FP8_NONE;
  constexpr int TK = P::TK, NST = P::NST, LPS = P::LPS, NG = P::NG, STAGE = P::STAGE;
  __shared__ __attribute__((aligned(1024))) unsigned char s_buf[NST * STAGE];
  __shared__ double s_red[3][4];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;      // 2 x 2 waves, 64 x 64 each
  const int r = lane & 31, g = lane >> 5;
  const int bm = blockIdx.x / a.tiles_n, bn = blockIdx.x - bm * a.tiles_n;
  const int m0 = bm * TM, n0 = bn * TN;

  // This lane's global source of each deposit slot at k = 0; advancing K adds a constant.
  const char* src[LPS];
#pragma unroll
  for (int s = 0; s < LPS; ++s) {
    const Slot sl = P::slot(s);
    const int c = (wave + 4 * sl.j) * 64 + lane;          // LDS chunk slot within the tile
    const int row = c / sl.C, kc = (c % sl.C) ^ swz(sl.C, row);
    const int rows = sl.is_w ? a.N : a.M;
    int grow = (sl.is_w ? n0 : m0) + row;
    grow = grow < rows ? grow : rows - 1;                 // rows past the edge repeat the last one (masked later)
    const char* base;
    int64_t row_bytes;
    switch (sl.kind) {
      case K_REF: base = reinterpret_cast<const char*>(sl.is_w ? a.w : a.x); row_bytes = (sl.is_w ? a.ldw : a.ldx) * 2; break;
      case K_GRID: base = reinterpret_cast<const char*>(sl.is_w ? a.wg : a.xg); row_bytes = static_cast<int64_t>(a.K) * 2; break;
      case K_I8: base = reinterpret_cast<const char*>(sl.is_w ? a.wi : a.xi); row_bytes = a.K; break;
      default: base = reinterpret_cast<const char*>(sl.is_w ? a.wf : a.xf); row_bytes = a.K; break;
    }
    src[s] = base + static_cast<int64_t>(grow) * row_bytes + kc * 16;
  }
  // Deposits [lo, hi) of this wave for stage kt.
  auto issue = [&](int kt, int lo, int hi) {
    unsigned char* st = s_buf + (kt % NST) * STAGE;
    const int64_t kb = static_cast<int64_t>(kt) * TK;     // k offset in elements
#pragma unroll
    for (int s = 0; s < LPS; ++s) {
      if (s < lo || s >= hi) continue;
      const Slot sl = P::slot(s);
      lds_deposit(src[s] + kb * (sl.kind <= K_GRID ? 2 : 1), st + sl.off + (wave + 4 * sl.j) * 1024);
    }
  };

  f32x16 acc_r[2][2];
  i32x16 acc_i[2][2];
  f32x16 acc_f[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) { acc_r[i][j][e] = 0.0f; acc_i[i][j][e] = 0; acc_f[i][j][e] = 0.0f; }

  // Fragment loads of one group: lane (r, g) supplies row r of a 32-row operand tile and
  // the g-th half of the instruction's K range, for A and B alike.  f[0..1] = A tiles,
  // f[2..3] = B tiles (the fp8 group needs two 16-byte chunks each: f[4..7]).
  auto load_group = [&](const unsigned char* st, int gi, i32x4 (&f)[8]) {
    const Group gr = P::group(gi);
    const int C = gr.kind <= K_GRID ? P::CB : P::CQ;
    const int ox = P::off_of(gr.kind, 0), ow = P::off_of(gr.kind, 1);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int ra = wm * 64 + i * 32 + r, rb = wn * 64 + i * 32 + r;
      if (gr.kind == K_F8) {
        f[i] = *reinterpret_cast<const i32x4*>(st + ox + chunk_off(C, ra, 2 * g));
        f[4 + i] = *reinterpret_cast<const i32x4*>(st + ox + chunk_off(C, ra, 2 * g + 1));
        f[2 + i] = *reinterpret_cast<const i32x4*>(st + ow + chunk_off(C, rb, 2 * g));
        f[6 + i] = *reinterpret_cast<const i32x4*>(st + ow + chunk_off(C, rb, 2 * g + 1));
      } else {
        f[i] = *reinterpret_cast<const i32x4*>(st + ox + chunk_off(C, ra, gr.ks * 2 + g));
        f[2 + i] = *reinterpret_cast<const i32x4*>(st + ow + chunk_off(C, rb, gr.ks * 2 + g));
      }
    }
  };
  auto run_group = [&](int gi, const i32x4 (&f)[8]) {
    const Group gr = P::group(gi);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (gr.kind == K_REF) {
          acc_r[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f[i]), __builtin_bit_cast(bf16x8, f[2 + j]), acc_r[i][j], 0, 0, 0);
        } else if (gr.kind == K_GRID) {
          acc_f[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f[i]), __builtin_bit_cast(bf16x8, f[2 + j]), acc_f[i][j], 0, 0, 0);
        } else if (gr.kind == K_I8) {
          acc_i[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f[i], f[2 + j], acc_i[i][j], 0, 0, 0);
        } else {
          i32x8 fa, fb;
#pragma unroll
          for (int e = 0; e < 4; ++e) { fa[e] = f[i][e]; fa[4 + e] = f[4 + i][e]; fb[e] = f[2 + j][e]; fb[4 + e] = f[6 + j][e]; }
          // format selectors 0 = E4M3 for both operands; block scales 2^0 (exponent byte 127)
          acc_f[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa, fb, acc_f[i][j], 0, 0, 0, 127, 0, 127);
        }
      }
  };

  const int KT = a.K / TK;
  // s_waitcnt immediates: vmcnt = n, expcnt / lgkmcnt unconstrained
  constexpr int WAIT_ALL = 0 | (7 << 4) | (15 << 8);
  constexpr int WAIT_BUT_ONE_STAGE = (LPS & 15) | (7 << 4) | (15 << 8) | ((LPS >> 4) << 14);
  issue(0, 0, LPS);
  if (NST == 3 && KT > 1) issue(1, 0, LPS);
  for (int kt = 0; kt < KT; ++kt) {
    // this wave's deposits of stage kt have landed (the stage after it may still be in flight)
    if (NST == 3 && kt + 1 < KT) __builtin_amdgcn_s_waitcnt(WAIT_BUT_ONE_STAGE);
    else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
    __builtin_amdgcn_s_barrier();      // ... and everyone's; also: all waves are done with stage kt-1
    asm volatile("" ::: "memory");     // LDS reads below must not move above the barrier
    const unsigned char* st = s_buf + (kt % NST) * STAGE;
    const bool more = kt + NST - 1 < KT;   // next deposits go into the buffer stage kt-1 just left

    // Software pipeline over the groups: fragments of group g+1 are requested before the
    // matrix instructions of group g are issued, and the stage's deposits are spread over
    // the groups so that the texture path works while the matrix cores do.
    i32x4 f[2][8];
    load_group(st, 0, f[0]);
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      if (gi + 1 < NG) load_group(st, gi + 1, f[(gi + 1) & 1]);
      if (more) issue(kt + NST - 1, gi * LPS / NG, (gi + 1) * LPS / NG);
      run_group(gi, f[gi & 1]);
    }
  }

  // ---- epilogue: squared differences in fp64.  Accumulator value e of a lane in one
  // 32x32 tile is output (row 8*(e/4) + 4*g + e%4, column lane%32) of that tile; rows and
  // columns past the matrix edge hold repeats of the last row and are skipped.
  const double sxi = DO_I8 ? static_cast<double>(*a.sx_i) : 0.0;
  const double sxf = DO_F8 ? static_cast<double>(*a.sx_f) : 0.0;
  double e_i = 0.0, e_f = 0.0, p = 0.0;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + j * 32 + r;
    const bool col_ok = n < a.N;
    const int ns = (a.w_per_channel && col_ok) ? n : 0;
    const double ci = DO_I8 ? sxi * static_cast<double>(a.sw_i[ns]) : 0.0;
    const double cf = DO_F8 ? sxf * static_cast<double>(a.sw_f[ns]) : 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * 64 + i * 32 + 8 * (e / 4) + 4 * g + (e % 4);
        const bool ok = col_ok && m < a.M;
        const double y = ok ? static_cast<double>(acc_r[i][j][e]) : 0.0;
        p = __builtin_fma(y, y, p);
        if constexpr (DO_I8) {
          const double q = ok ? static_cast<double>(acc_i[i][j][e]) : 0.0;
          const double d = __builtin_fma(-ci, q, y);
          e_i = __builtin_fma(d, d, e_i);
        }
        if constexpr (DO_F8) {
          const double q = ok ? static_cast<double>(acc_f[i][j][e]) : 0.0;
          const double d = __builtin_fma(-cf, q, y);
          e_f = __builtin_fma(d, d, e_f);
        }
      }
  }
  e_i = wave_sum(e_i);
  e_f = wave_sum(e_f);
  p = wave_sum(p);
  if (lane == 0) { s_red[0][wave] = e_i; s_red[1][wave] = e_f; s_red[2][wave] = p; }
  __syncthreads();
  if (tid == 0) {
    if (a.part_i) a.part_i[blockIdx.x] = (s_red[0][0] + s_red[0][1]) + (s_red[0][2] + s_red[0][3]);
    if (a.part_f) a.part_f[blockIdx.x] = (s_red[1][0] + s_red[1][1]) + (s_red[1][2] + s_red[1][3]);
    a.part_p[blockIdx.x] = (s_red[2][0] + s_red[2][1]) + (s_red[2][2] + s_red[2][3]);
  }
}

}  // namespace

int wa_gemm_blocks(int64_t M, int64_t N) {
  return static_cast<int>(((M + TM - 1) / TM) * ((N + TN - 1) / TN));
}

int launch_wa_gemm(const WaGemmParams& p, hipStream_t st) {
  if (p.K % 64 != 0) return MOFQ_ERR_UNSUPPORTED;
  GemmArgs a{};
  a.x = static_cast<const uint16_t*>(p.x); a.ldx = p.ldx;
  a.w = static_cast<const uint16_t*>(p.w); a.ldw = p.ldw;
  a.xi = p.xi; a.wi = p.wi; a.xf = p.xf; a.wf = p.wf;
  a.xg = static_cast<const uint16_t*>(p.xg); a.wg = static_cast<const uint16_t*>(p.wg);
  a.sx_i = p.sx_i; a.sw_i = p.sw_i; a.sx_f = p.sx_f; a.sw_f = p.sw_f;
  a.w_per_channel = p.w_per_channel;
  a.M = static_cast<int32_t>(p.M); a.N = static_cast<int32_t>(p.N); a.K = static_cast<int32_t>(p.K);
  a.tiles_n = static_cast<int32_t>((p.N + TN - 1) / TN);
  a.part_i = p.part_i; a.part_f = p.part_f; a.part_p = p.part_p;
  const dim3 grid(static_cast<unsigned>(wa_gemm_blocks(p.M, p.N)));
  const bool di = p.xi != nullptr;
  const int f8 = p.xg ? FP8_EXACT : (p.xf ? FP8_NATIVE : FP8_NONE);
#define MOFQ_WA(DI, F8) \
  if (di == DI && f8 == F8) hipLaunchKernelGGL((wa_gemm_kernel<DI, F8>), grid, dim3(256), 0, st, a);
  if (!di && f8 == FP8_NONE) return MOFQ_ERR_INVALID_ARG;
  MOFQ_WA(true, FP8_NONE) MOFQ_WA(true, FP8_NATIVE) MOFQ_WA(true, FP8_EXACT)
  MOFQ_WA(false, FP8_NATIVE) MOFQ_WA(false, FP8_EXACT)
#undef MOFQ_WA
  return hip_status(hipGetLastError());
}

}  // namespace mofq
