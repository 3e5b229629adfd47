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
};

constexpr int kTensorBlocks = 1024;  // partial results of per-tensor passes

// Enqueue the scale search.  Returns a mofq_status_t.
int launch_sweep(const SweepParams& p, hipStream_t stream);

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
};
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
  mofq_qout_t out;
};
int launch_emit(const EmitParams& p, hipStream_t stream);

inline int hip_status(hipError_t e) { return e == hipSuccess ? MOFQ_OK : MOFQ_ERR_HIP; }

}  // namespace mofq
