// Host-side internal interface between the C ABI (mofq_api.hip) and the kernel
// launchers.  Not part of the public boundary.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mofq.h"

namespace mofq {

constexpr int kMaxFmt = 2;  // formats scored together in one sweep launch

// Per-unit results of a sweep for up to kMaxFmt formats (device arrays of
// `units` entries each; slot f belongs to fmt[f]).
struct UnitRecords {
  float* scale[kMaxFmt];
  int32_t* clip[kMaxFmt];
  double* err[kMaxFmt];
  double* energy;  // sum x^2 per unit
};

struct SweepParams {
  const void* w;
  int32_t dtype;
  int64_t rows, cols, ld;
  int32_t gran, group;
  int32_t scale_f16;
  int32_t n_clip;
  int32_t n_fmt;          // 1 or 2
  int32_t fmt[kMaxFmt];   // formats, same bit-width
  float clip[MOFQ_MAX_CLIP];
  UnitRecords rec;
  // per-tensor granularity only:
  float* absmax_part;     // [kTensorBlocks]
  double* sse_part;       // [kTensorBlocks][n_fmt][n_clip]
  double* energy_part;    // [kTensorBlocks]
  const float* ext_absmax;  // device, one value, or nullptr: use this magnitude instead of the tensor's own
  // per-tensor (INT8, FP8-E4M3) pair with one clip ratio only: the scoring pass also writes
  // the quantized tensor in both formats (dense rows), saving two further reads of the input
  uint8_t* emit_i8;         // int8 codes, or nullptr
  void* emit_f8;            // e4m3 codes (1 byte) or grid values as bf16 (2 bytes)
  int32_t emit_f8_as_bf16;
  // per-channel pair of two different formats (bf16 input) with one clip ratio only: the pass
  // also writes the grid values of format slot f as bf16, dense [rows][cols], to emit_grid[f]
  void* emit_grid[kMaxFmt];
};

constexpr int kTensorBlocks = 1024;  // partial results of per-tensor passes

// max|x| of a tensor folded into a running maximum: *running = max(*running, max|x|).
// `absmax_part` / `energy_part` are scratch of kTensorBlocks entries.
int launch_running_absmax(const SweepParams& p, float* running, hipStream_t stream);

// Enqueue the scale search.  Returns a mofq_status_t.
int launch_sweep(const SweepParams& p, hipStream_t stream);
// Sort-based search for per-channel 4-bit searches on 16-bit inputs; returns
// MOFQ_ERR_UNSUPPORTED (nothing enqueued) outside that domain.
int launch_sweep_sorted(const SweepParams& p, hipStream_t stream);
// The same for up to kSweepGroupMax tensors of one row length, dtype and configuration in one
// launch (MOFQ_ERR_UNSUPPORTED, nothing enqueued, if they differ or are outside the domain).
constexpr int kSweepGroupMax = 8;
int launch_sweep_sorted_group(const SweepParams* p, int n, hipStream_t stream);
// Scale search of n tensors: one launch where launch_sweep_sorted_group takes them, else one
// launch_sweep per tensor.
int launch_sweep_group(const SweepParams* p, int n, hipStream_t stream);

// Tensor-level reduce + Algorithm 1's strict-less select over n_cand formats
// whose unit errors live in `err[c]` (units entries each).
struct DecideParams {
  int64_t units;
  int32_t n_cand;
  const double* err[MOFQ_MAX_CANDIDATES];
  const double* energy;          // [units] or nullptr
  mofq_result_t* result;         // device
  double* tensor_err_out;        // optional: err of candidate 0 (device) or nullptr
  double* energy_out;            // optional (device) or nullptr
  double* part;                  // optional scratch, (MOFQ_MAX_CANDIDATES + 1) * kDecideBlocks doubles:
                                 // with it, many units are first reduced by kDecideBlocks workgroups
};
constexpr int kDecideBlocks = 256;
int launch_decide(const DecideParams& p, hipStream_t stream);

// Emit codes and per-unit outputs for the format chosen in *result (or slot 0 if
// result is null).
struct EmitParams {
  const void* w;
  int32_t dtype;
  int64_t rows, cols, ld;
  int32_t gran, group;
  int32_t scale_f16_out;
  int32_t n_cand;
  int32_t fmt[MOFQ_MAX_CANDIDATES];
  const float* scale[MOFQ_MAX_CANDIDATES];
  const int32_t* clip[MOFQ_MAX_CANDIDATES];
  const double* err[MOFQ_MAX_CANDIDATES];
  const mofq_result_t* result;   // device, may be nullptr (then candidate 0)
  const uint8_t* unit_fmt;       // device [units] or nullptr: candidate index per unit (overrides result)
  mofq_qout_t out;
  int32_t as_bf16_values;        // 8-bit formats: out.codes receives the grid values as bf16
  int32_t max_blocks;            // 0: fill the device; else a cap for emission that runs beside other kernels
};
int launch_emit(const EmitParams& p, hipStream_t stream);

// Tensor-level reduce + select + the per-unit outputs of the winner for several tensors in
// one launch (one workgroup per tensor): the small dependent steps between the search and
// the code emission, batched so that a model-wide pass does not pay their latency per
// tensor.  Every tensor must have at most kFinishMaxUnits units.
struct FinishParams {
  DecideParams d;
  int32_t scale_f16_out;
  const float* scale[MOFQ_MAX_CANDIDATES];
  const int32_t* clip[MOFQ_MAX_CANDIDATES];
  void* out_scales;          // may be nullptr
  int32_t* out_clip;         // may be nullptr
  double* out_unit_err;      // may be nullptr
};
constexpr int kFinishBatch = 12;
constexpr int64_t kFinishMaxUnits = 16 * 1024;
int launch_finish_batch(const FinishParams* p, int n, hipStream_t stream);

// Per unit: the first candidate with the strictly smallest error; writes its index and
// its error.
struct PickUnitsParams {
  int64_t units;
  int32_t n_cand;
  const double* err[MOFQ_MAX_CANDIDATES];
  uint8_t* unit_fmt;     // [units]
  double* picked_err;    // [units]
};
int launch_pick_units(const PickUnitsParams& p, hipStream_t stream);

// Layer-output error of one linear layer: partial sums per 128x128 output tile.
// A null xi/wi (or xf/wf) pair skips that format.
// One quantized product of the layer-output kernel: sum_i Gx[t,i] * Gw[o,i], scaled by
// sx * sw[o] in the reduction.  Operand arrays are dense ([M][K] and [N][K]).
enum WaKind : int32_t {
  WA_NONE = 0,
  WA_GRID_BF16 = 1,   // grid values stored as bf16 (exact), bf16 matrix cores
  WA_INT8 = 2,        // int8 codes, int8 matrix cores
  WA_FP8 = 3,         // e4m3 codes, fp8 matrix cores
};
struct WaProduct {
  int32_t kind;
  const void* x; const void* w;
  const float* sx;                 // device, one value; nullptr = 1 (unquantized input)
  const float* sw;                 // device, 1 or N values
  double* part;                    // [wa_gemm_blocks(M, N)] squared-difference partials
  // optional second part of the same product (same scales): grid values as bf16, dense
  // [M][kWaSideCols] and [N][kWaSideCols], multiplied on the bf16 matrix cores and added
  const void* xs; const void* ws;
};
struct WaGemmParams {
  const void* x; int64_t ldx;      // bf16 [M][K]
  const void* w; int64_t ldw;      // bf16 [N][K]
  WaProduct q[2];                  // up to two quantized products (kind WA_NONE = unused)
  int32_t w_per_channel;
  int64_t M, N, K;
  double* part_p;                  // [wa_gemm_blocks(M, N)] sum of Y^2
};
int wa_gemm_blocks(int64_t M, int64_t N);
int launch_wa_gemm(const WaGemmParams& p, hipStream_t stream);

// The fused weight-activation path (both 8-bit formats as candidates, per-tensor scales)
// works on groups of up to kWaGroup layers: one launch per step for the whole group.
constexpr int kWaGroup = 8;

// Pass 1 + 2 over the inputs of the group's layers (up to 2 * kWaGroup tensors, one launch per
// pass): largest magnitude, then both quantized copies and the tensor error of each format.
// A tensor with data == nullptr is skipped (an activation that the previous layer already
// prepared).  The tensor error is left as partial sums over wa_prep_segments() fixed pieces of
// the tensor.
// With the E4M3 codes going to the fp8 matrix cores, the activation's columns of outstanding
// magnitude (outlier channels, Section 3.2) are split off: inside one matrix instruction the
// unit aligns the 8 products of a group of 8 consecutive k to the largest of them and drops
// what falls below its window, so a group that holds an outlier column loses bits of its
// other products.  The split-off columns (at most kWaSideCols) are zeroed in the activation
// operand of the fp8 product and their share of the sum, X[:, cols] W[:, cols]^T, is added by one
// K step on the bf16 matrix cores from the grid values (exact): the same sum, without the loss.
constexpr int kWaSideCols = 64;
struct WaPrepTensor {
  const void* data;          // bf16 [rows][cols], rows `ld` elements apart
  int64_t rows, cols, ld;
  float ratio;               // clip ratio of the scale (1 for activations)
  float* absmax_part;        // [kTensorBlocks]
  double* sse_part;          // [wa_prep_segments(rows, cols)][2]: INT8, E4M3
  uint8_t* q_i8;             // [rows][cols] int8 codes, dense
  uint8_t* q_f8;             // [rows][cols] e4m3 codes, dense
  uint8_t* q_g;              // [rows][cols] e4m3 grid values as bf16, dense; or nullptr
  float* scale;              // [2]: INT8 scale, E4M3 scale
  // column split for the fp8-unit product (all null otherwise)
  int32_t is_x;              // activation: picks the columns; weight: uses its activation's pick
  float* colmax;             // X: [cols] scratch, largest magnitude per column
  uint8_t* col_slot;         // [cols]: slot of a split-off column, 0xFF otherwise (X writes, W reads its X's)
  int32_t* side_cols;        // [kWaSideCols + 1]: the split-off columns in ascending order, then their number
  uint8_t* q_f8_main;        // X: [rows][cols] e4m3 codes with the split-off columns zeroed, dense
  uint16_t* side;            // [rows][kWaSideCols] bf16: e4m3 grid values at the split-off columns, zero beyond their number
};
int wa_prep_segments(int64_t rows, int64_t cols);
int launch_wa_prep(const WaPrepTensor* t, int n, hipStream_t stream);

// After the matrix kernels of a group: per layer (one workgroup each) the fixed-order sums of
// its per-tile partials, Algorithm 1's select, the result record, and the one-unit outputs
// (scale, clip index 0, tensor error) of the chosen format for both tensors.
struct WaFinishTensor {
  int32_t n_segments;        // 0: no outputs for this tensor
  const double* sse_part;    // as written by launch_wa_prep
  const float* scale;
  void* out_scales;          // one float; may be nullptr
  int32_t* out_clip;         // may be nullptr
  double* out_unit_err;      // may be nullptr
};
struct WaFinishParams {
  DecideParams d;                          // err[c] = the tile partials of candidate c's format
  int32_t fmt_slot[MOFQ_MAX_CANDIDATES];   // per candidate: 0 INT8, 1 E4M3
  WaFinishTensor t[2];                     // X, W
};
int launch_wa_finish(const WaFinishParams* p, int n, hipStream_t stream);

// Codes of the chosen format into the caller's buffers, for the layers of a group in one
// launch: a copy of the quantized operand the matrix kernel used (no second quantization).
// Where the chosen format's codes already sit in the destination (src == dst) nothing is moved.
struct WaCopyTensor {
  const uint8_t* src[2];     // INT8 codes, E4M3 codes
  uint8_t* dst;              // nullptr: nothing to do
  int64_t bytes;             // multiple of 16
};
struct WaCopyParams {
  const mofq_result_t* result;
  int32_t n_cand;
  int32_t fmt_slot[MOFQ_MAX_CANDIDATES];
  WaCopyTensor t[2];
};
int launch_wa_copy(const WaCopyParams* p, int n, hipStream_t stream);

inline int hip_status(hipError_t e) { return e == hipSuccess ? MOFQ_OK : MOFQ_ERR_HIP; }

}  // namespace mofq
