// Micro-kernels that measure what the part in front of us sustains: a plain device copy, a
// register-only vector FMA loop (fp32 and fp64) and register-only matrix-core loops for the
// three operand types of the layer-output kernel.  A harness times them with events around the
// launch and prints the rates beside its roofline fractions, so that a fraction of the
// published peak can be read against what the device really delivers.  Nothing here is on
// the quantization path.
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

constexpr int kThreads = 256;

// dst[i] = src[i] for n 16-byte chunks, grid-stride, four chunks in flight per lane
__global__ __launch_bounds__(kThreads) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  for (; i + 3 * stride < n; i += 4 * stride) {
    const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < n; i += stride) dst[i] = src[i];
}

// sink[thread] = xor of the n 16-byte chunks the thread visits (grid-stride, eight in flight): a
// pass that only reads, like the scoring kernels
__global__ __launch_bounds__(kThreads) void read_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ sink, int64_t n) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + 7 * stride < n; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(&src[i + u * stride]);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  for (; i < n; i += stride) acc ^= src[i];
  if (acc[0] == 0x12345678u && acc[1] == 0x9ABCDEF0u && acc[2] == 1u && acc[3] == 2u)   // practically never: keeps the loads alive
    sink[static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x] = acc;
}

// kChains independent fused multiply-add chains per lane, `iters` rounds: 2 flop per chain and
// round.  The multiplier is below 1 in magnitude, so the values stay finite; the result is
// stored so that the loop cannot be dropped.
constexpr int kChains = 16;
template <typename T>
__global__ __launch_bounds__(kThreads) void fma_kernel(T* sink, int iters, T mul, T add) {
  T v[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c) v[c] = static_cast<T>(threadIdx.x + c);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kChains; ++c) {
      if constexpr (sizeof(T) == 4) v[c] = __builtin_fmaf(v[c], mul, add);
      else v[c] = __builtin_fma(v[c], mul, add);
    }
  }
  T s = 0;
#pragma unroll
  for (int c = 0; c < kChains; ++c) s += v[c];
  sink[static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x] = s;
}

// Four independent 32x32 accumulator tiles per wave, `iters` rounds of one matrix instruction
// each; operands are constant registers (values do not matter for the rate).
constexpr int kTiles = 4;
template <int KIND>   // WA_GRID_BF16: bf16, WA_INT8: int8, WA_FP8: e4m3 through the scaled f8f6f4 form
__global__ __launch_bounds__(kThreads) void mfma_kernel(float* sink, int iters) {
  using acc_t = typename std::conditional<KIND == WA_INT8, i32x16, f32x16>::type;
  acc_t acc[kTiles];
#pragma unroll
  for (int t = 0; t < kTiles; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0;
  i32x4 a4, b4;
  i32x8 a8, b8;
#pragma unroll
  for (int e = 0; e < 4; ++e) {   // bf16 1.0 twice per register, or four int8 ones
    a4[e] = KIND == WA_INT8 ? 0x01010101 : 0x3F803F80;
    b4[e] = a4[e];
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { a8[e] = 0x38383838; b8[e] = 0x38383838; }   // e4m3 1.0
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < kTiles; ++t) {
      if constexpr (KIND == WA_GRID_BF16)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a4), __builtin_bit_cast(bf16x8, b4), acc[t], 0, 0, 0);
      else if constexpr (KIND == WA_INT8)
        acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a4, b4, acc[t], 0, 0, 0);
      else
        acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[t], 0, 0, 0, 127, 0, 127);
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int t = 0; t < kTiles; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += static_cast<float>(acc[t][e]);
  sink[static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x] = s;
}

}  // namespace

}  // namespace mofq

using namespace mofq;

extern "C" int mofq_device_ceiling(int32_t kind, void* scratch, size_t scratch_bytes, int32_t iters,
                                   double* work, void* stream) {
  if (!scratch || !work || iters < 1 || (reinterpret_cast<uintptr_t>(scratch) & 15u)) return MOFQ_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return MOFQ_ERR_HIP;
  const int blocks = cus * 8;                              // 8 workgroups of 4 waves per compute unit
  const size_t sink_bytes = static_cast<size_t>(blocks) * kThreads * sizeof(double);
  switch (kind) {
    case MOFQ_CEILING_COPY: {
      const int64_t n = static_cast<int64_t>(scratch_bytes / 32);   // 16-byte chunks per half
      if (n < 1) return MOFQ_ERR_WORKSPACE;
      const u32x4* src = static_cast<const u32x4*>(scratch);
      for (int i = 0; i < iters; ++i)
        hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(kThreads), 0, st, src, const_cast<u32x4*>(src) + n, n);
      *work = 32.0 * static_cast<double>(n) * iters;         // bytes read + bytes written
      break;
    }
    case MOFQ_CEILING_READ: {
      // the first sink_bytes * 2 hold the (practically never written) sink, the rest is read
      if (scratch_bytes < 4 * sink_bytes) return MOFQ_ERR_WORKSPACE;
      char* base = static_cast<char*>(scratch);
      const int64_t n = static_cast<int64_t>((scratch_bytes - 2 * sink_bytes) / 16);
      for (int i = 0; i < iters; ++i)
        hipLaunchKernelGGL(read_kernel, dim3(blocks), dim3(kThreads), 0, st,
                           reinterpret_cast<const u32x4*>(base + 2 * sink_bytes), reinterpret_cast<u32x4*>(base), n);
      *work = 16.0 * static_cast<double>(n) * iters;         // bytes read
      break;
    }
    case MOFQ_CEILING_FMA_F32:
      if (scratch_bytes < sink_bytes) return MOFQ_ERR_WORKSPACE;
      hipLaunchKernelGGL(fma_kernel<float>, dim3(blocks), dim3(kThreads), 0, st, static_cast<float*>(scratch), iters, 0.999f, 0.5f);
      *work = 2.0 * kChains * static_cast<double>(iters) * blocks * kThreads;
      break;
    case MOFQ_CEILING_FMA_F64:
      if (scratch_bytes < sink_bytes) return MOFQ_ERR_WORKSPACE;
      hipLaunchKernelGGL(fma_kernel<double>, dim3(blocks), dim3(kThreads), 0, st, static_cast<double*>(scratch), iters, 0.999, 0.5);
      *work = 2.0 * kChains * static_cast<double>(iters) * blocks * kThreads;
      break;
    case MOFQ_CEILING_MFMA_BF16:
      if (scratch_bytes < sink_bytes) return MOFQ_ERR_WORKSPACE;
      hipLaunchKernelGGL(mfma_kernel<WA_GRID_BF16>, dim3(blocks), dim3(kThreads), 0, st, static_cast<float*>(scratch), iters);
      *work = 2.0 * 32 * 32 * 16 * kTiles * static_cast<double>(iters) * blocks * (kThreads / 64);
      break;
    case MOFQ_CEILING_MFMA_INT8:
      if (scratch_bytes < sink_bytes) return MOFQ_ERR_WORKSPACE;
      hipLaunchKernelGGL(mfma_kernel<WA_INT8>, dim3(blocks), dim3(kThreads), 0, st, static_cast<float*>(scratch), iters);
      *work = 2.0 * 32 * 32 * 32 * kTiles * static_cast<double>(iters) * blocks * (kThreads / 64);
      break;
    case MOFQ_CEILING_MFMA_FP8:
      if (scratch_bytes < sink_bytes) return MOFQ_ERR_WORKSPACE;
      hipLaunchKernelGGL(mfma_kernel<WA_FP8>, dim3(blocks), dim3(kThreads), 0, st, static_cast<float*>(scratch), iters);
      *work = 2.0 * 32 * 32 * 64 * kTiles * static_cast<double>(iters) * blocks * (kThreads / 64);
      break;
    default:
      return MOFQ_ERR_INVALID_ARG;
  }
  return hip_status(hipGetLastError());
}
