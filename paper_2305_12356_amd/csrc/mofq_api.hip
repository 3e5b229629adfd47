// The C ABI: argument validation, workspace carving and the order of launches.
// No device memory is allocated here and nothing synchronises.
#include <algorithm>
#include <cstring>
#include <mutex>

#include "mofq_internal.h"

using namespace mofq;

namespace {

constexpr size_t kAlign = 256;

bool is4(int f) { return f == MOFQ_INT4 || f == MOFQ_FP4_E2M1 || f == MOFQ_FP4_E2M1_IEEE; }
bool is8(int f) { return f == MOFQ_INT8 || f == MOFQ_FP8_E4M3 || f == MOFQ_FP8_E5M2; }
// format pairs the search kernels score in one launch (one read of the tensor)
bool paired(int a, int b) {
  return (a == MOFQ_INT4 && b == MOFQ_FP4_E2M1) || (a == MOFQ_FP4_E2M1 && b == MOFQ_INT4) ||
         (a == MOFQ_INT8 && b == MOFQ_FP8_E4M3) || (a == MOFQ_FP8_E4M3 && b == MOFQ_INT8);
}
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Compute units of the current device (256 on an MI355X); 256 when no device answers, so that
// the host-only planning calls work anywhere.
int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    return 256;
  }
  return n;
}


int check_tensor(const mofq_tensor_t* t) {
  if (!t || !t->data) return MOFQ_ERR_INVALID_ARG;
  if (t->rows <= 0 || t->cols <= 0 || t->ld < t->cols) return MOFQ_ERR_INVALID_ARG;
  if (t->dtype != MOFQ_F32 && t->dtype != MOFQ_F16 && t->dtype != MOFQ_BF16) return MOFQ_ERR_INVALID_ARG;
  if (!aligned16(t->data) || t->cols % 8 != 0 || t->ld % 8 != 0) return MOFQ_ERR_MISALIGNED;
  return MOFQ_OK;
}

int check_cfg(const mofq_tensor_t* t, const mofq_scale_cfg_t* c) {
  if (!c || !c->clip_ratios) return MOFQ_ERR_INVALID_ARG;
  if (c->n_clip < 1 || c->n_clip > MOFQ_MAX_CLIP) return MOFQ_ERR_INVALID_ARG;
  if (c->scale_dtype != MOFQ_F32 && c->scale_dtype != MOFQ_F16) return MOFQ_ERR_INVALID_ARG;
  for (int k = 0; k < c->n_clip; ++k)
    if (!(c->clip_ratios[k] > 0.0f) || !(c->clip_ratios[k] <= 1.0f)) return MOFQ_ERR_INVALID_ARG;
  switch (c->gran) {
    case MOFQ_PER_TENSOR:
      return MOFQ_OK;
    case MOFQ_PER_CHANNEL:
      if (t->cols > 32768) return MOFQ_ERR_UNSUPPORTED;
      return MOFQ_OK;
    case MOFQ_PER_GROUP:
      if (c->group_size != 32 && c->group_size != 64 && c->group_size != 128 && c->group_size != 256)
        return MOFQ_ERR_UNSUPPORTED;
      if (t->cols % c->group_size != 0) return MOFQ_ERR_UNSUPPORTED;
      return MOFQ_OK;
  }
  return MOFQ_ERR_INVALID_ARG;
}

int check_out(const mofq_qout_t* o, bool need_codes) {
  if (!o) return MOFQ_ERR_INVALID_ARG;
  if (need_codes && (!o->codes || !o->scales)) return MOFQ_ERR_INVALID_ARG;
  if (!aligned16(o->codes) || !aligned16(o->scales) || !aligned16(o->clip_idx) || !aligned16(o->unit_err))
    return MOFQ_ERR_MISALIGNED;
  return MOFQ_OK;
}

// Bump allocator over the caller's workspace.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  template <typename T> T* take(size_t n) {
    off = (off + kAlign - 1) / kAlign * kAlign;
    T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    return r;
  }
};

struct WOnlyWs {
  float* scale[MOFQ_MAX_CANDIDATES];
  int32_t* clip[MOFQ_MAX_CANDIDATES];
  double* err[MOFQ_MAX_CANDIDATES];
  double* energy;
  float* absmax_part;
  double* sse_part;
  double* energy_part;
  double* decide_part;
  size_t bytes;
};

WOnlyWs carve_w_only(void* ws, int64_t units, int n_cand, int gran, int n_clip) {
  Carver c(ws);
  WOnlyWs w{};
  for (int i = 0; i < n_cand; ++i) {
    w.scale[i] = c.take<float>(units);
    w.clip[i] = c.take<int32_t>(units);
    w.err[i] = c.take<double>(units);
  }
  w.energy = c.take<double>(units);
  w.decide_part = c.take<double>(static_cast<size_t>(MOFQ_MAX_CANDIDATES + 1) * kDecideBlocks);
  if (gran == MOFQ_PER_TENSOR) {
    w.absmax_part = c.take<float>(kTensorBlocks);
    w.energy_part = c.take<double>(kTensorBlocks);
    w.sse_part = c.take<double>(static_cast<size_t>(kTensorBlocks) * kMaxFmt * n_clip);
  }
  w.bytes = (c.off + kAlign - 1) / kAlign * kAlign;
  return w;
}

// Scale search of all candidates (two formats per launch), results in the workspace.
// Optional outputs of the scoring pass itself (per-tensor (INT8, FP8-E4M3) pair only).
struct SweepEmit {
  uint8_t* i8;
  void* f8;
  int f8_as_bf16;
  void* grid[2];   // per-channel pair: bf16 grid values of candidate 0 and candidate 1
};

// Parameters of the launch that scores candidates c0 .. c0 + n - 1 (n = 2: a pair of different
// formats that share one read of the tensor).  A launch takes at most kMaxFmt formats.
int sweep_params(const mofq_tensor_t* t, const int32_t* cand, int c0, int n,
                 const mofq_scale_cfg_t* cfg, const WOnlyWs& w, SweepParams* out) {
  if (n < 1 || n > kMaxFmt || c0 < 0 || c0 + n > MOFQ_MAX_CANDIDATES) return MOFQ_ERR_INVALID_ARG;
  SweepParams p{};
  p.w = t->data;
  p.dtype = t->dtype;
  p.rows = t->rows;
  p.cols = t->cols;
  p.ld = t->ld;
  p.gran = cfg->gran;
  p.group = cfg->group_size;
  p.scale_f16 = cfg->scale_dtype == MOFQ_F16;
  p.n_clip = cfg->n_clip;
  std::memcpy(p.clip, cfg->clip_ratios, sizeof(float) * cfg->n_clip);
  p.n_fmt = n;
  // kernels exist for the (INT, FP) order; a reversed pair swaps its record slots
  int slot[2] = {c0, c0 + 1};
  if (n == 2 && !(cand[c0] == MOFQ_INT4 || cand[c0] == MOFQ_INT8)) std::swap(slot[0], slot[1]);
  for (int f = 0; f < n; ++f) {
    p.fmt[f] = cand[slot[f]];
    p.rec.scale[f] = w.scale[slot[f]];
    p.rec.clip[f] = w.clip[slot[f]];
    p.rec.err[f] = w.err[slot[f]];
  }
  p.rec.energy = (c0 == 0) ? w.energy : nullptr;
  p.absmax_part = w.absmax_part;
  p.sse_part = w.sse_part;
  p.energy_part = w.energy_part;
  *out = p;
  return MOFQ_OK;
}

// The whole candidate list is one launch: a single format or a pair of different ones.
bool one_sweep_launch(const int32_t* cand, int n_cand) {
  return n_cand == 1 || (n_cand == 2 && paired(cand[0], cand[1]));
}

int sweep_candidates(const mofq_tensor_t* t, const int32_t* cand, int n_cand,
                     const mofq_scale_cfg_t* cfg, const WOnlyWs& w, hipStream_t st,
                     const float* ext_absmax = nullptr, const SweepEmit* em = nullptr) {
  int c0 = 0;
  while (c0 < n_cand) {
    // two different formats share one launch (one read of the tensor); a repeated
    // format is scored on its own
    const int n = (c0 + 1 < n_cand && paired(cand[c0], cand[c0 + 1])) ? 2 : 1;
    SweepParams p{};
    int rc = sweep_params(t, cand, c0, n, cfg, w, &p);
    if (rc != MOFQ_OK) return rc;
    p.ext_absmax = ext_absmax;
    if (em) {
      if (n != 2) return MOFQ_ERR_INVALID_ARG;
      p.emit_i8 = em->i8;
      p.emit_f8 = em->f8;
      p.emit_f8_as_bf16 = em->f8_as_bf16;
      // launch slots are in (INT, FP) order whatever the candidates' order
      const bool swapped = p.fmt[0] != cand[c0];
      p.emit_grid[0] = em->grid[swapped ? 1 : 0];
      p.emit_grid[1] = em->grid[swapped ? 0 : 1];
    }
    rc = launch_sweep(p, st);
    if (rc != MOFQ_OK) return rc;
    c0 += n;
  }
  return MOFQ_OK;
}

int check_candidates(const int32_t* cand, int n) {
  if (!cand || n < 1 || n > MOFQ_MAX_CANDIDATES) return MOFQ_ERR_INVALID_ARG;
  for (int i = 0; i < n; ++i) {
    if (!is4(cand[i]) && !is8(cand[i])) return MOFQ_ERR_INVALID_ARG;
    if (is4(cand[i]) != is4(cand[0])) return MOFQ_ERR_INVALID_ARG;  // one bit-width per call
  }
  return MOFQ_OK;
}


// ---- weight-activation (layer-output metric) ------------------------------------

const float kOne = 1.0f;

mofq_scale_cfg_t x_cfg() {   // activations: per-tensor, no clip search (Section 3.2)
  mofq_scale_cfg_t c{};
  c.gran = MOFQ_PER_TENSOR;
  c.group_size = 0;
  c.scale_dtype = MOFQ_F32;
  c.n_clip = 1;
  c.clip_ratios = &kOne;
  return c;
}

int check_wa(const mofq_tensor_t* w, const mofq_tensor_t* x, const int32_t* cand, int n_cand,
             const mofq_scale_cfg_t* w_cfg) {
  int rc = check_tensor(x);
  if (rc) return rc;
  if (x->cols != w->cols) return MOFQ_ERR_INVALID_ARG;
  for (int c = 0; c < n_cand; ++c)
    if (cand[c] != MOFQ_INT8 && cand[c] != MOFQ_FP8_E4M3) return MOFQ_ERR_UNSUPPORTED;   // the low-bit matmul units
  if (w->dtype != MOFQ_BF16 || x->dtype != MOFQ_BF16) return MOFQ_ERR_UNSUPPORTED;
  if (w_cfg->n_clip != 1 || w_cfg->scale_dtype != MOFQ_F32) return MOFQ_ERR_UNSUPPORTED;
  if (w_cfg->gran != MOFQ_PER_TENSOR && w_cfg->gran != MOFQ_PER_CHANNEL) return MOFQ_ERR_UNSUPPORTED;
  if (w->cols % 64 != 0) return MOFQ_ERR_UNSUPPORTED;
  if (w->rows > (1 << 30) || x->rows > (1 << 30) || w->cols > 32768) return MOFQ_ERR_UNSUPPORTED;
  return MOFQ_OK;
}

struct WaWs {
  WOnlyWs xrec, wrec;
  uint8_t* xq[2];   // [0] INT8 codes, [1] E4M3 codes (fp8-unit mode) or bf16 grid values
  uint8_t* wq[2];
  double* part[3];  // INT8 error, E4M3 error, reference energy; one value per output tile
  int blocks;
  size_t bytes;
};

WaWs carve_wa(void* ws, const mofq_tensor_t* w, const mofq_tensor_t* x, int n_cand, int w_gran) {
  WaWs a{};
  const int64_t units_w = mofq_num_units(w->rows, w->cols, w_gran, 0);
  a.xrec = carve_w_only(ws, 1, n_cand, MOFQ_PER_TENSOR, 1);
  char* base = static_cast<char*>(ws);
  size_t off = a.xrec.bytes;
  a.wrec = carve_w_only(base ? base + off : nullptr, units_w, n_cand, w_gran, 1);
  off += a.wrec.bytes;
  Carver c(base ? base + off : nullptr);
  for (int f = 0; f < 2; ++f) {
    a.xq[f] = c.take<uint8_t>(static_cast<size_t>(x->rows) * x->cols * (f ? 2 : 1));
    a.wq[f] = c.take<uint8_t>(static_cast<size_t>(w->rows) * w->cols * (f ? 2 : 1));
  }
  a.blocks = wa_gemm_blocks(x->rows, w->rows);
  for (int i = 0; i < 3; ++i) a.part[i] = c.take<double>(a.blocks);
  a.bytes = off + (c.off + kAlign - 1) / kAlign * kAlign;
  return a;
}

// ---- weight-only select with the layer-output error (Section 4.1: tensor error or
// layer-output error suffices for the weight-only case).  The input stays in 16 bits; each
// candidate's weights are quantized as in the tensor-error path (scales searched by
// tensor error), and the kernel compares X W^T with s[o] * (X G^T).
int check_wo_output(const mofq_tensor_t* w, const mofq_tensor_t* x, const int32_t* cand, int n_cand,
                    const mofq_scale_cfg_t* w_cfg) {
  int rc = check_tensor(x);
  if (rc) return rc;
  if (x->cols != w->cols) return MOFQ_ERR_INVALID_ARG;
  if (n_cand > 2) return MOFQ_ERR_UNSUPPORTED;                 // two quantized products per launch
  if (w->dtype != MOFQ_BF16 || x->dtype != MOFQ_BF16) return MOFQ_ERR_UNSUPPORTED;
  if (x->ld != x->cols) return MOFQ_ERR_UNSUPPORTED;            // X is also the dense operand of the quantized products
  if (w_cfg->gran != MOFQ_PER_TENSOR && w_cfg->gran != MOFQ_PER_CHANNEL) return MOFQ_ERR_UNSUPPORTED;
  if (w->cols % 64 != 0) return MOFQ_ERR_UNSUPPORTED;
  if (w->rows > (1 << 30) || x->rows > (1 << 30) || w->cols > 32768) return MOFQ_ERR_UNSUPPORTED;
  return MOFQ_OK;
}

struct WoOutWs {
  WOnlyWs wrec;
  uint8_t* wg[2];   // grid values of W per candidate, bf16, dense
  double* part[3];  // error per candidate, reference energy; one value per output tile
  int blocks;
  size_t bytes;
};

WoOutWs carve_wo_output(void* ws, const mofq_tensor_t* w, const mofq_tensor_t* x, int n_cand,
                        const mofq_scale_cfg_t* cfg) {
  WoOutWs a{};
  const int64_t units_w = mofq_num_units(w->rows, w->cols, cfg->gran, 0);
  a.wrec = carve_w_only(ws, units_w, n_cand, cfg->gran, cfg->n_clip);
  char* base = static_cast<char*>(ws);
  Carver c(base ? base + a.wrec.bytes : nullptr);
  for (int f = 0; f < n_cand; ++f) a.wg[f] = c.take<uint8_t>(static_cast<size_t>(w->rows) * w->cols * 2);
  a.blocks = wa_gemm_blocks(x->rows, w->rows);
  for (int i = 0; i < 3; ++i) a.part[i] = c.take<double>(a.blocks);
  a.bytes = a.wrec.bytes + (c.off + kAlign - 1) / kAlign * kAlign;
  return a;
}

int wo_output_score(const mofq_tensor_t* w, const mofq_tensor_t* x, const int32_t* cand, int n_cand,
                    const mofq_scale_cfg_t* w_cfg, const WoOutWs& a, hipStream_t st,
                    hipEvent_t ev0, hipEvent_t ev1) {
  int rc;
  // A pair of different formats with per-channel absmax scales (one clip ratio): the scoring pass
  // holds each row in registers and writes both candidates' grid values itself.
  const bool fused = n_cand == 2 && paired(cand[0], cand[1]) && w_cfg->gran == MOFQ_PER_CHANNEL && w_cfg->n_clip == 1;
  const SweepEmit em{nullptr, nullptr, 0, {a.wg[0], a.wg[1]}};
  if ((rc = sweep_candidates(w, cand, n_cand, w_cfg, a.wrec, st, nullptr, fused ? &em : nullptr))) return rc;
  WaGemmParams g{};
  for (int c = 0; c < n_cand; ++c) {
    if (!fused) {
      EmitParams e{};
      e.w = w->data;
      e.dtype = w->dtype;
      e.rows = w->rows;
      e.cols = w->cols;
      e.ld = w->ld;
      e.gran = w_cfg->gran;
      e.group = 0;
      e.n_cand = 1;
      e.fmt[0] = cand[c];
      e.scale[0] = a.wrec.scale[c];
      e.clip[0] = a.wrec.clip[c];
      e.err[0] = a.wrec.err[c];
      e.result = nullptr;
      e.out.codes = a.wg[c];
      e.as_bf16_values = 1;
      if ((rc = launch_emit(e, st))) return rc;
    }
    g.q[c].kind = WA_GRID_BF16;
    g.q[c].x = x->data;          // the unquantized input, scale 1
    g.q[c].w = a.wg[c];
    g.q[c].sx = nullptr;
    g.q[c].sw = a.wrec.scale[c];
    g.q[c].part = a.part[c];
  }
  g.x = x->data; g.ldx = x->ld;
  g.w = w->data; g.ldw = w->ld;
  g.w_per_channel = w_cfg->gran == MOFQ_PER_CHANNEL;
  g.M = x->rows; g.N = w->rows; g.K = w->cols;
  g.part_p = a.part[2];
  if (ev0 && hipEventRecord(ev0, st) != hipSuccess) return MOFQ_ERR_HIP;
  if ((rc = launch_wa_gemm(g, st))) return rc;
  if (ev1 && hipEventRecord(ev1, st) != hipSuccess) return MOFQ_ERR_HIP;
  return MOFQ_OK;
}

// Quantize X and W in every candidate format, then one pass over the matrix cores
// that leaves per-tile partial errors in the workspace.
// Work on a second stream of the caller beside `main`: fork() orders the side stream after
// what is on `main` so far, join() makes `main` wait for the side stream.  The two events live
// for one call (destroying an event with waits pending is deferred by the runtime).  Without a
// second stream (null, or the same as `main`) everything stays on `main`.
struct SideWork {
  hipStream_t main, side;
  bool two, forked = false;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  SideWork(hipStream_t m, void* s) : main(m), side(static_cast<hipStream_t>(s)), two(s != nullptr && s != m) {
    if (!two) side = main;
  }
  SideWork(const SideWork&) = delete;
  SideWork& operator=(const SideWork&) = delete;
  ~SideWork() {
    if (ev_fork) (void)hipEventDestroy(ev_fork);
    if (ev_join) (void)hipEventDestroy(ev_join);
  }
  int init() {
    if (!two) return MOFQ_OK;
    if (hipEventCreateWithFlags(&ev_fork, hipEventDisableTiming) != hipSuccess) return MOFQ_ERR_HIP;
    if (hipEventCreateWithFlags(&ev_join, hipEventDisableTiming) != hipSuccess) return MOFQ_ERR_HIP;
    return MOFQ_OK;
  }
  int fork() {
    if (!two) return MOFQ_OK;
    if (hipEventRecord(ev_fork, main) != hipSuccess || hipStreamWaitEvent(side, ev_fork, 0) != hipSuccess)
      return MOFQ_ERR_HIP;
    forked = true;
    return MOFQ_OK;
  }
  // returns `status`, or the join's own failure if `status` was fine
  int join(int status) {
    if (!forked) return status;
    forked = false;
    if (hipEventRecord(ev_join, side) != hipSuccess || hipStreamWaitEvent(main, ev_join, 0) != hipSuccess)
      return status ? status : static_cast<int>(MOFQ_ERR_HIP);
    return status;
  }
};

int wa_score(const mofq_tensor_t* w, const mofq_tensor_t* x, const int32_t* cand, int n_cand,
             const mofq_scale_cfg_t* w_cfg, bool fp8_unit, const WaWs& a, hipStream_t st,
             hipEvent_t ev0, hipEvent_t ev1) {
  const mofq_scale_cfg_t xc = x_cfg();
  int rc;
  // With both formats as candidates, a per-tensor scoring pass also writes both quantized
  // copies of its tensor (one read instead of three).
  bool both = false;
  if (n_cand == 2)
    both = (cand[0] == MOFQ_INT8 && cand[1] == MOFQ_FP8_E4M3) || (cand[0] == MOFQ_FP8_E4M3 && cand[1] == MOFQ_INT8);
  const bool fused_x = both, fused_w = both && w_cfg->gran == MOFQ_PER_TENSOR;
  const SweepEmit ex{a.xq[0], a.xq[1], fp8_unit ? 0 : 1, {nullptr, nullptr}}, ew{a.wq[0], a.wq[1], fp8_unit ? 0 : 1, {nullptr, nullptr}};
  if ((rc = sweep_candidates(x, cand, n_cand, &xc, a.xrec, st, nullptr, fused_x ? &ex : nullptr))) return rc;
  if ((rc = sweep_candidates(w, cand, n_cand, w_cfg, a.wrec, st, nullptr, fused_w ? &ew : nullptr))) return rc;
  WaGemmParams g{};
  int n_q = 0;
  for (int f = 0; f < 2; ++f) {
    const int fmt = f == 0 ? MOFQ_INT8 : MOFQ_FP8_E4M3;
    int slot = -1;
    for (int c = n_cand - 1; c >= 0; --c)
      if (cand[c] == fmt) slot = c;
    if (slot < 0) continue;
    for (int which = 0; which < 2; ++which) {   // 0: X, 1: W
      if (which ? fused_w : fused_x) continue;  // already written by the scoring pass
      const mofq_tensor_t* t = which ? w : x;
      const WOnlyWs& rec = which ? a.wrec : a.xrec;
      EmitParams e{};
      e.w = t->data;
      e.dtype = t->dtype;
      e.rows = t->rows;
      e.cols = t->cols;
      e.ld = t->ld;
      e.gran = which ? w_cfg->gran : MOFQ_PER_TENSOR;
      e.group = 0;
      e.n_cand = 1;
      e.fmt[0] = fmt;
      e.scale[0] = rec.scale[slot];
      e.clip[0] = rec.clip[slot];
      e.err[0] = rec.err[slot];
      e.result = nullptr;
      e.out.codes = which ? a.wq[f] : a.xq[f];
      e.as_bf16_values = (f == 1 && !fp8_unit);
      if ((rc = launch_emit(e, st))) return rc;
    }
    WaProduct& q = g.q[n_q++];
    q.kind = f == 0 ? WA_INT8 : (fp8_unit ? WA_FP8 : WA_GRID_BF16);
    q.x = a.xq[f];
    q.w = a.wq[f];
    q.sx = a.xrec.scale[slot];
    q.sw = a.wrec.scale[slot];
    q.part = a.part[f];
  }
  g.x = x->data; g.ldx = x->ld;
  g.w = w->data; g.ldw = w->ld;
  g.w_per_channel = w_cfg->gran == MOFQ_PER_CHANNEL;
  g.M = x->rows; g.N = w->rows; g.K = w->cols;
  g.part_p = a.part[2];
  if (ev0 && hipEventRecord(ev0, st) != hipSuccess) return MOFQ_ERR_HIP;
  if ((rc = launch_wa_gemm(g, st))) return rc;
  if (ev1 && hipEventRecord(ev1, st) != hipSuccess) return MOFQ_ERR_HIP;
  return MOFQ_OK;
}

// Algorithm 1's loop body for one layer with the layer-output metric, any candidate list and
// per-tensor or per-channel weight scales: the general path (one launch per step).
int select_wa_general(const mofq_tensor_t* w, const mofq_tensor_t* x, const int32_t* candidates,
                      int n_candidates, int metric, const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out,
                      const mofq_qout_t* x_out, mofq_result_t* result, void* ws, size_t ws_bytes,
                      hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  int rc;
  const WaWs a = carve_wa(ws, w, x, n_candidates, w_cfg->gran);
  if (!ws || ws_bytes < a.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  if ((rc = wa_score(w, x, candidates, n_candidates, w_cfg,
                     metric == MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT, a, st, ev0, ev1)))
    return rc;
  DecideParams d{};
  d.units = a.blocks;
  d.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) d.err[c] = candidates[c] == MOFQ_INT8 ? a.part[0] : a.part[1];
  d.energy = a.part[2];
  d.result = result;
  if ((rc = launch_decide(d, st))) return rc;
  // second quantize_layer call of Algorithm 1: W and X in the chosen format
  for (int which = 0; which < 2; ++which) {
    const mofq_tensor_t* t = which ? w : x;
    const mofq_qout_t* o = which ? w_out : x_out;
    if (!o) continue;
    const WOnlyWs& rec = which ? a.wrec : a.xrec;
    EmitParams e{};
    e.w = t->data;
    e.dtype = t->dtype;
    e.rows = t->rows;
    e.cols = t->cols;
    e.ld = t->ld;
    e.gran = which ? w_cfg->gran : MOFQ_PER_TENSOR;
    e.group = 0;
    e.n_cand = n_candidates;
    for (int c = 0; c < n_candidates; ++c) {
      e.fmt[c] = candidates[c];
      e.scale[c] = rec.scale[c];
      e.clip[c] = rec.clip[c];
      e.err[c] = rec.err[c];
    }
    e.result = result;
    e.out = *o;
    if ((rc = launch_emit(e, st))) return rc;
  }
  return MOFQ_OK;
}

// ---- the fused weight-activation path ----------------------------------------------------
// INT8 against FP8-E4M3 with per-tensor weight scales (the configuration of Section 5's
// W8A8 experiments).  Per layer: the two quantize passes over X and W together
// (launch_wa_prep), the matrix kernel, one small kernel for select + one-unit outputs, and a
// copy of the chosen codes.  The weight's E4M3 codes are written straight into the caller's
// code buffer by the quantize pass (they are an operand of the fp8-unit product, and the
// output itself if E4M3 is chosen); if INT8 is chosen its codes are copied over them.  An
// activation that the previous layer of the call already used (same descriptor: the q/k/v
// or gate/up projections of a block) is quantized once.
bool wa_fused(const int32_t* cand, int n_cand, const mofq_scale_cfg_t* w_cfg) {
  return n_cand == 2 && w_cfg->gran == MOFQ_PER_TENSOR && cand[0] != cand[1] &&
         (cand[0] == MOFQ_INT8 || cand[0] == MOFQ_FP8_E4M3) && (cand[1] == MOFQ_INT8 || cand[1] == MOFQ_FP8_E4M3);
}

struct WaFusedTensorWs {
  uint8_t* i8;
  uint8_t* f8;
  uint8_t* g;
  float* absmax_part;
  double* sse_part;
  float* scale;
  // fp8-unit product: the column split (see WaPrepTensor); null for the exact product
  uint8_t* f8_main;
  float* colmax;
  uint8_t* col_slot;
  int32_t* side_cols;
  uint16_t* side;
};
// Workspace of one layer: the quantized operands and records of X and W, and the per-tile
// partials of the matrix kernel (INT8 error, E4M3 error, reference energy).
struct WaLayerWs {
  WaFusedTensorWs x, w;
  double* part[3];
  bool fresh_x;   // false: x is the previous layer's (same descriptor, same group)
};

// The layers are worked off in groups of up to kWaGroup consecutive layers holding up to
// kWaGroupElems weight elements (a decoder block of the 7B shape is one group): with a second
// stream a whole group is prepared while the previous group is multiplied, so that the two
// streams meet once per group and not once per layer.  Returns the number of layers of the
// group that starts at i0.
constexpr int64_t kWaGroupElems = int64_t{1} << 28;
int wa_group_length(int n_layers, const mofq_tensor_t* w, int i0) {
  int64_t elems = 0;
  int n = 0;
  for (; i0 + n < n_layers && n < kWaGroup; ++n) {
    const int64_t e = w[i0 + n].rows * w[i0 + n].cols;
    if (n > 0 && elems + e > kWaGroupElems) break;
    elems += e;
  }
  return n;
}

bool wa_same_x(const mofq_tensor_t* x, int i) {
  return x[i].data == x[i - 1].data && x[i].rows == x[i - 1].rows && x[i].cols == x[i - 1].cols &&
         x[i].ld == x[i - 1].ld;
}

// Carves the workspaces of layers [i0, i0 + n) out of `arena` (null: sizes only); returns the bytes.
size_t carve_wa_group(void* arena, int i0, int n, const mofq_tensor_t* w, const mofq_tensor_t* x, bool exact,
                      WaLayerWs* out) {
  Carver c(arena);
  for (int j = 0; j < n; ++j) {
    const int i = i0 + j;
    WaLayerWs l{};
    l.fresh_x = j == 0 || !wa_same_x(x, i);
    for (int which = 0; which < 2; ++which) {
      WaFusedTensorWs& t = which ? l.w : l.x;
      if (!which && !l.fresh_x) {
        if (out) t = out[j - 1].x;
        continue;
      }
      const size_t e = static_cast<size_t>(which ? w[i].rows * w[i].cols : x[i].rows * x[i].cols);
      t.i8 = c.take<uint8_t>(e);
      t.f8 = which ? nullptr : c.take<uint8_t>(e);   // the weight's live in the caller's code buffer
      t.g = exact ? c.take<uint8_t>(2 * e) : nullptr;
      t.absmax_part = c.take<float>(kTensorBlocks);
      t.sse_part = c.take<double>(2 * kTensorBlocks);
      t.scale = c.take<float>(2);
      if (!exact) {
        const size_t rows = static_cast<size_t>(which ? w[i].rows : x[i].rows);
        t.side = c.take<uint16_t>(rows * kWaSideCols);
        if (!which) {
          const size_t cols = static_cast<size_t>(x[i].cols);
          t.f8_main = c.take<uint8_t>(e);
          t.colmax = c.take<float>(cols);
          t.col_slot = c.take<uint8_t>(cols);
          t.side_cols = c.take<int32_t>(kWaSideCols + 1);
        }
      }
    }
    for (int q = 0; q < 3; ++q) l.part[q] = c.take<double>(wa_gemm_blocks(x[i].rows, w[i].rows));
    if (out) out[j] = l;
  }
  return (c.off + kAlign - 1) / kAlign * kAlign;
}

// One arena, large enough for any group: the groups follow each other on one stream.
size_t wa_fused_bytes(int n_layers, const mofq_tensor_t* w, const mofq_tensor_t* x, bool exact) {
  size_t bytes = 0;
  for (int i0 = 0, n = 0; i0 < n_layers; i0 += n) {
    n = wa_group_length(n_layers, w, i0);
    bytes = std::max(bytes, carve_wa_group(nullptr, i0, n, w, x, exact, nullptr));
  }
  return bytes;
}

// Arguments are validated by the caller except for the workspace.  x_out may be null (no
// activation outputs), ev_begin / ev_end may be null.
int select_layers_wa(int n_layers, const mofq_tensor_t* w, const mofq_tensor_t* x, const int32_t* cand,
                     int n_cand, int metric, const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out,
                     const mofq_qout_t* x_out, mofq_result_t* results, void* ws, size_t ws_bytes,
                     hipStream_t st, void* const* ev_begin, void* const* ev_end) {
  int rc;
  auto ev = [](void* const* list, int i) { return list ? static_cast<hipEvent_t>(list[i]) : nullptr; };
  if (!wa_fused(cand, n_cand, w_cfg)) {
    for (int i = 0; i < n_layers; ++i)
      if ((rc = select_wa_general(&w[i], &x[i], cand, n_cand, metric, w_cfg, &w_out[i], x_out ? &x_out[i] : nullptr,
                                  &results[i], ws, ws_bytes, st, ev(ev_begin, i), ev(ev_end, i))))
        return rc;
    return MOFQ_OK;
  }
  const bool fp8_unit = metric == MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT;
  if (!ws || ws_bytes < wa_fused_bytes(n_layers, w, x, !fp8_unit) || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  int fmt_slot[MOFQ_MAX_CANDIDATES] = {0, 0, 0, 0};
  for (int c = 0; c < n_cand; ++c) fmt_slot[c] = cand[c] == MOFQ_FP8_E4M3;

  // the group's layers are [i0, i0 + n), their workspaces l[0 .. n)
  auto prep = [&](int i0, int n, const WaLayerWs* l, hipStream_t s) {
    WaPrepTensor t[2 * kWaGroup] = {};
    for (int j = 0; j < n; ++j) {
      const int i = i0 + j;
      WaPrepTensor& px = t[2 * j];
      WaPrepTensor& pw = t[2 * j + 1];
      if (l[j].fresh_x) {
        px.data = x[i].data; px.rows = x[i].rows; px.cols = x[i].cols; px.ld = x[i].ld;
        px.ratio = 1.0f;   // activations: per tensor at the full range (Section 3.2)
        px.absmax_part = l[j].x.absmax_part; px.sse_part = l[j].x.sse_part;
        px.q_i8 = l[j].x.i8; px.q_f8 = l[j].x.f8; px.q_g = l[j].x.g; px.scale = l[j].x.scale;
        px.is_x = 1;
        px.colmax = l[j].x.colmax; px.col_slot = l[j].x.col_slot; px.side_cols = l[j].x.side_cols;
        px.q_f8_main = l[j].x.f8_main; px.side = l[j].x.side;
      }
      pw.data = w[i].data; pw.rows = w[i].rows; pw.cols = w[i].cols; pw.ld = w[i].ld;
      pw.ratio = w_cfg->clip_ratios[0];
      pw.absmax_part = l[j].w.absmax_part; pw.sse_part = l[j].w.sse_part;
      pw.q_i8 = l[j].w.i8; pw.q_f8 = static_cast<uint8_t*>(w_out[i].codes); pw.q_g = l[j].w.g;
      pw.scale = l[j].w.scale;
      // the weight's side operand follows its activation's pick of columns
      pw.is_x = 0;
      pw.col_slot = l[j].x.col_slot; pw.side_cols = l[j].x.side_cols; pw.side = l[j].w.side;
    }
    return launch_wa_prep(t, 2 * n, s);
  };
  auto products = [&](int i0, int n, const WaLayerWs* l) {
    int r;
    for (int j = 0; j < n; ++j) {
      const int i = i0 + j;
      WaGemmParams g{};
      g.q[0].kind = WA_INT8;
      g.q[0].x = l[j].x.i8; g.q[0].w = l[j].w.i8;
      g.q[0].sx = l[j].x.scale; g.q[0].sw = l[j].w.scale;
      g.q[0].part = l[j].part[0];
      g.q[1].kind = fp8_unit ? WA_FP8 : WA_GRID_BF16;
      g.q[1].x = fp8_unit ? l[j].x.f8_main : l[j].x.g;
      g.q[1].xs = fp8_unit ? l[j].x.side : nullptr;
      g.q[1].ws = fp8_unit ? l[j].w.side : nullptr;
      g.q[1].w = fp8_unit ? static_cast<const uint8_t*>(w_out[i].codes) : l[j].w.g;
      g.q[1].sx = l[j].x.scale + 1; g.q[1].sw = l[j].w.scale + 1;
      g.q[1].part = l[j].part[1];
      g.x = x[i].data; g.ldx = x[i].ld;
      g.w = w[i].data; g.ldw = w[i].ld;
      g.w_per_channel = 0;
      g.M = x[i].rows; g.N = w[i].rows; g.K = w[i].cols;
      g.part_p = l[j].part[2];
      if (ev(ev_begin, i) && hipEventRecord(ev(ev_begin, i), st) != hipSuccess) return static_cast<int>(MOFQ_ERR_HIP);
      if ((r = launch_wa_gemm(g, st))) return r;
      if (ev(ev_end, i) && hipEventRecord(ev(ev_end, i), st) != hipSuccess) return static_cast<int>(MOFQ_ERR_HIP);
    }
    WaFinishParams f[kWaGroup] = {};
    for (int j = 0; j < n; ++j) {
      const int i = i0 + j;
      f[j].d.units = wa_gemm_blocks(x[i].rows, w[i].rows);
      f[j].d.n_cand = n_cand;
      for (int c = 0; c < n_cand; ++c) { f[j].d.err[c] = l[j].part[fmt_slot[c]]; f[j].fmt_slot[c] = fmt_slot[c]; }
      f[j].d.energy = l[j].part[2];
      f[j].d.result = &results[i];
      if (x_out) {
        f[j].t[0].n_segments = wa_prep_segments(x[i].rows, x[i].cols);
        f[j].t[0].sse_part = l[j].x.sse_part; f[j].t[0].scale = l[j].x.scale;
        f[j].t[0].out_scales = x_out[i].scales; f[j].t[0].out_clip = x_out[i].clip_idx;
        f[j].t[0].out_unit_err = x_out[i].unit_err;
      }
      f[j].t[1].n_segments = wa_prep_segments(w[i].rows, w[i].cols);
      f[j].t[1].sse_part = l[j].w.sse_part; f[j].t[1].scale = l[j].w.scale;
      f[j].t[1].out_scales = w_out[i].scales; f[j].t[1].out_clip = w_out[i].clip_idx;
      f[j].t[1].out_unit_err = w_out[i].unit_err;
    }
    return launch_wa_finish(f, n, st);
  };
  auto codes = [&](int i0, int n, const WaLayerWs* l, hipStream_t s) {
    WaCopyParams p[kWaGroup] = {};
    for (int j = 0; j < n; ++j) {
      const int i = i0 + j;
      p[j].result = &results[i];
      p[j].n_cand = n_cand;
      for (int c = 0; c < n_cand; ++c) p[j].fmt_slot[c] = fmt_slot[c];
      if (x_out) {
        p[j].t[0].src[0] = l[j].x.i8; p[j].t[0].src[1] = l[j].x.f8;
        p[j].t[0].dst = static_cast<uint8_t*>(x_out[i].codes);
        p[j].t[0].bytes = x[i].rows * x[i].cols;
      }
      p[j].t[1].src[0] = l[j].w.i8; p[j].t[1].src[1] = static_cast<const uint8_t*>(w_out[i].codes);
      p[j].t[1].dst = static_cast<uint8_t*>(w_out[i].codes);
      p[j].t[1].bytes = w[i].rows * w[i].cols;
    }
    return launch_wa_copy(p, n, s);
  };

  // Group by group on the caller's stream: the quantize passes, the matrix kernels, the selects,
  // the code copies.  (Running the passes of the next group on a second stream beside the matrix
  // kernels was measured and lost: two waves of 216-240 registers on every SIMD leave no room
  // for a second kernel's waves, so the side work only delays the matrix kernels.)
  WaLayerWs cur[kWaGroup];
  for (int i0 = 0, n = 0; i0 < n_layers; i0 += n) {
    n = wa_group_length(n_layers, w, i0);
    carve_wa_group(ws, i0, n, w, x, !fp8_unit, cur);
    if ((rc = prep(i0, n, cur, st))) return rc;
    if ((rc = products(i0, n, cur))) return rc;
    if ((rc = codes(i0, n, cur, st))) return rc;
  }
  return MOFQ_OK;
}

// Algorithm 1's loop body for one weight tensor with the tensor-error metric: search every
// candidate, reduce + select on the device, emit the winner.  Arguments are already validated
// except for the workspace.
int select_w_only(const mofq_tensor_t* w, const int32_t* candidates, int n_candidates,
                  const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out, mofq_result_t* result,
                  void* ws, size_t ws_bytes, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  int rc;
  const int64_t units = mofq_num_units(w->rows, w->cols, w_cfg->gran, w_cfg->group_size);
  const WOnlyWs s = carve_w_only(ws, units, n_candidates, w_cfg->gran, w_cfg->n_clip);
  if (!ws || ws_bytes < s.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  if (ev0 && hipEventRecord(ev0, st) != hipSuccess) return MOFQ_ERR_HIP;
  if ((rc = sweep_candidates(w, candidates, n_candidates, w_cfg, s, st))) return rc;
  if (ev1 && hipEventRecord(ev1, st) != hipSuccess) return MOFQ_ERR_HIP;
  DecideParams d{};
  d.units = units;
  d.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) d.err[c] = s.err[c];
  d.energy = s.energy;
  d.part = s.decide_part;
  d.result = result;
  if ((rc = launch_decide(d, st))) return rc;
  EmitParams e{};
  e.w = w->data;
  e.dtype = w->dtype;
  e.rows = w->rows;
  e.cols = w->cols;
  e.ld = w->ld;
  e.gran = w_cfg->gran;
  e.group = w_cfg->group_size;
  e.scale_f16_out = w_cfg->scale_dtype == MOFQ_F16;
  e.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) {
    e.fmt[c] = candidates[c];
    e.scale[c] = s.scale[c];
    e.clip[c] = s.clip[c];
    e.err[c] = s.err[c];
  }
  e.result = result;
  e.out = *w_out;
  return launch_emit(e, st);
}

}  // namespace

// ---- the workspace of mofq_select_layer_static ------------------------------------------
// One array per GPU, in the library's own device image, so that the call needs no allocation
// and no workspace argument.  In host code the array's name is only a handle for the symbol
// lookup, never a device address: the address is asked for once per device (with that device
// current) and kept, and kernels, like everything else on the host side, get that pointer.
static __device__ __align__(256) unsigned char scratch[MOFQ_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MOFQ_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return MOFQ_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return MOFQ_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MOFQ_OK;
}

}  // namespace

extern "C" {

int64_t mofq_num_units(int64_t rows, int64_t cols, int32_t gran, int32_t group_size) {
  if (rows <= 0 || cols <= 0) return -1;
  switch (gran) {
    case MOFQ_PER_TENSOR: return 1;
    case MOFQ_PER_CHANNEL: return rows;
    case MOFQ_PER_GROUP:
      if (group_size <= 0 || cols % group_size != 0) return -1;
      return rows * (cols / group_size);
  }
  return -1;
}

const char* mofq_status_string(int status) {
  switch (status) {
    case MOFQ_OK: return "ok";
    case MOFQ_ERR_INVALID_ARG: return "invalid argument";
    case MOFQ_ERR_UNSUPPORTED: return "unsupported dtype / granularity / shape combination";
    case MOFQ_ERR_MISALIGNED: return "pointer not 16-byte aligned or cols/ld not a multiple of 8";
    case MOFQ_ERR_WORKSPACE: return "workspace too small";
    case MOFQ_ERR_HIP: return "HIP launch failed";
  }
  return "unknown status";
}

size_t mofq_workspace_bytes(const mofq_tensor_t* w, const mofq_tensor_t* x, int32_t n_candidates,
                            int32_t metric, const mofq_scale_cfg_t* w_cfg) {
  if (!w || !w_cfg || n_candidates < 1 || n_candidates > MOFQ_MAX_CANDIDATES) return 0;
  const int64_t units = mofq_num_units(w->rows, w->cols, w_cfg->gran, w_cfg->group_size);
  if (units <= 0 || w_cfg->n_clip < 1 || w_cfg->n_clip > MOFQ_MAX_CLIP) return 0;
  if (metric == MOFQ_ERR_TENSOR && !x)
    return carve_w_only(nullptr, units, n_candidates, w_cfg->gran, w_cfg->n_clip).bytes;
  if ((metric == MOFQ_ERR_LAYER_OUTPUT || metric == MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT) && x &&
      x->rows > 0 && x->cols == w->cols &&
      (w_cfg->gran == MOFQ_PER_TENSOR || w_cfg->gran == MOFQ_PER_CHANNEL)) {
    // the larger of the general path's need and, where it can apply, the fused path's
    size_t b = carve_wa(nullptr, w, x, n_candidates, w_cfg->gran).bytes;
    if (n_candidates == 2 && w_cfg->gran == MOFQ_PER_TENSOR)
      b = std::max(b, wa_fused_bytes(1, w, x, metric == MOFQ_ERR_LAYER_OUTPUT));
    return b;
  }
  if (metric == MOFQ_ERR_LAYER_OUTPUT_W_ONLY && x && x->rows > 0 && x->cols == w->cols && n_candidates <= 2 &&
      (w_cfg->gran == MOFQ_PER_TENSOR || w_cfg->gran == MOFQ_PER_CHANNEL))
    return carve_wo_output(nullptr, w, x, n_candidates, w_cfg).bytes;
  return 0;
}

int mofq_quantize(const mofq_tensor_t* t, int32_t format, const mofq_scale_cfg_t* cfg,
                  const mofq_qout_t* out, double* tensor_err, void* ws, size_t ws_bytes,
                  void* stream) {
  int rc = check_tensor(t);
  if (rc) return rc;
  if ((rc = check_cfg(t, cfg))) return rc;
  if ((rc = check_out(out, true))) return rc;
  if ((rc = check_candidates(&format, 1))) return rc;
  const int64_t units = mofq_num_units(t->rows, t->cols, cfg->gran, cfg->group_size);
  const WOnlyWs w = carve_w_only(ws, units, 1, cfg->gran, cfg->n_clip);
  if (!ws || ws_bytes < w.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = sweep_candidates(t, &format, 1, cfg, w, st))) return rc;
  if (tensor_err) {
    DecideParams d{};
    d.units = units;
    d.n_cand = 1;
    d.err[0] = w.err[0];
    d.part = w.decide_part;
    d.tensor_err_out = tensor_err;
    if ((rc = launch_decide(d, st))) return rc;
  }
  EmitParams e{};
  e.w = t->data;
  e.dtype = t->dtype;
  e.rows = t->rows;
  e.cols = t->cols;
  e.ld = t->ld;
  e.gran = cfg->gran;
  e.group = cfg->group_size;
  e.scale_f16_out = cfg->scale_dtype == MOFQ_F16;
  e.n_cand = 1;
  e.fmt[0] = format;
  e.scale[0] = w.scale[0];
  e.clip[0] = w.clip[0];
  e.err[0] = w.err[0];
  e.result = nullptr;
  e.out = *out;
  return launch_emit(e, st);
}

int mofq_score(const mofq_tensor_t* w, const mofq_tensor_t* x, int32_t format, int32_t metric,
               const mofq_scale_cfg_t* w_cfg, double* err, double* ref_energy, void* ws,
               size_t ws_bytes, void* stream) {
  int rc = check_tensor(w);
  if (rc) return rc;
  if ((rc = check_cfg(w, w_cfg))) return rc;
  if ((rc = check_candidates(&format, 1))) return rc;
  if (!err) return MOFQ_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (metric == MOFQ_ERR_TENSOR) {
    if (x) return MOFQ_ERR_INVALID_ARG;
    const int64_t units = mofq_num_units(w->rows, w->cols, w_cfg->gran, w_cfg->group_size);
    const WOnlyWs s = carve_w_only(ws, units, 1, w_cfg->gran, w_cfg->n_clip);
    if (!ws || ws_bytes < s.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
    if ((rc = sweep_candidates(w, &format, 1, w_cfg, s, st))) return rc;
    DecideParams d{};
    d.units = units;
    d.n_cand = 1;
    d.err[0] = s.err[0];
    d.energy = s.energy;
    d.part = s.decide_part;
    d.tensor_err_out = err;
    d.energy_out = ref_energy;
    return launch_decide(d, st);
  }
  if (metric == MOFQ_ERR_LAYER_OUTPUT_W_ONLY) {
    if (!x) return MOFQ_ERR_INVALID_ARG;
    if ((rc = check_wo_output(w, x, &format, 1, w_cfg))) return rc;
    const WoOutWs a = carve_wo_output(ws, w, x, 1, w_cfg);
    if (!ws || ws_bytes < a.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
    if ((rc = wo_output_score(w, x, &format, 1, w_cfg, a, st, nullptr, nullptr))) return rc;
    DecideParams d{};
    d.units = a.blocks;
    d.n_cand = 1;
    d.err[0] = a.part[0];
    d.energy = a.part[2];
    d.tensor_err_out = err;
    d.energy_out = ref_energy;
    return launch_decide(d, st);
  }
  if (metric == MOFQ_ERR_LAYER_OUTPUT || metric == MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT) {
    if (!x) return MOFQ_ERR_INVALID_ARG;
    if ((rc = check_wa(w, x, &format, 1, w_cfg))) return rc;
    const WaWs a = carve_wa(ws, w, x, 1, w_cfg->gran);
    if (!ws || ws_bytes < a.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
    if ((rc = wa_score(w, x, &format, 1, w_cfg, metric == MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT, a, st,
                       nullptr, nullptr)))
      return rc;
    DecideParams d{};
    d.units = a.blocks;
    d.n_cand = 1;
    d.err[0] = format == MOFQ_INT8 ? a.part[0] : a.part[1];
    d.energy = a.part[2];
    d.tensor_err_out = err;
    d.energy_out = ref_energy;
    return launch_decide(d, st);
  }
  return MOFQ_ERR_INVALID_ARG;
}

}  // extern "C"

namespace {

// A batch of mofq_select_layers ends at kFinishBatch tensors or once it holds 2 MB of input per
// compute unit.  The batch is the unit of overlap (its select and emission run beside the next
// batch's searches) and of search grouping (its tensors of one row length share a launch), so
// it should span the same-length tensors of a transformer block; past that, larger batches
// only lengthen the exposed emission of the last one.  Measured on 256 compute units with the
// 7B-shaped set, whole pass: 31.4 ms at 256 MB, 30.6 ms at 400 MB, 30.3 ms at 520 MB.  The budget is
// per compute unit because what it balances, a launch that fills the device against the
// exposed tail, scales with the device.  Returns the number of tensors in the batch that
// starts at i0.
int batch_length(int n_layers, const mofq_tensor_t* w, int i0, int cus) {
  const int64_t batch_bytes = static_cast<int64_t>(cus) * (int64_t{2} << 20);
  int64_t bytes = 0;
  int nb = 0;
  for (; i0 + nb < n_layers && nb < kFinishBatch; ++nb) {
    const int64_t b = w[i0 + nb].rows * w[i0 + nb].cols * (w[i0 + nb].dtype == MOFQ_F32 ? 4 : 2);
    if (nb > 0 && bytes + b > batch_bytes) break;
    bytes += b;
  }
  return nb;
}

// Tensors of a batch with one row length and dtype share a search launch (up to
// kSweepGroupMax of them, adjacent or not: a larger launch fills the device better than
// several small ones, and nothing orders the searches inside a batch).  first[j] (j < nb)
// receives the batch-relative index of the first member of tensor j's launch.
void plan_search_groups(const mofq_tensor_t* w, int nb, const int32_t* cand, int n_cand, int* first) {
  const bool joinable = one_sweep_launch(cand, n_cand);
  for (int j = 0; j < nb; ++j) first[j] = -1;
  for (int j = 0; j < nb; ++j) {
    if (first[j] >= 0) continue;
    first[j] = j;
    int n = 1;
    for (int k = j + 1; joinable && k < nb && n < kSweepGroupMax; ++k)
      if (first[k] < 0 && w[k].cols == w[j].cols && w[k].dtype == w[j].dtype) {
        first[k] = j;
        ++n;
      }
  }
}

}  // namespace

extern "C" {

int mofq_select_layers_search_groups(int32_t n_layers, const mofq_tensor_t* w, const int32_t* candidates,
                                     int32_t n_candidates, int32_t* group_first) {
  if (n_layers < 1 || !w || !group_first) return MOFQ_ERR_INVALID_ARG;
  const int rc = check_candidates(candidates, n_candidates);
  if (rc) return rc;
  const int cus = compute_units();
  for (int i0 = 0, nb = 0; i0 < n_layers; i0 += nb) {
    nb = batch_length(n_layers, w, i0, cus);
    int first[kFinishBatch];
    plan_search_groups(w + i0, nb, candidates, n_candidates, first);
    for (int j = 0; j < nb; ++j) group_first[i0 + j] = i0 + first[j];
  }
  return MOFQ_OK;
}

size_t mofq_select_layers_workspace_bytes(int32_t n_layers, const mofq_tensor_t* w,
                                          int32_t n_candidates, const mofq_scale_cfg_t* w_cfg) {
  if (n_layers < 1 || !w) return 0;
  size_t total = 0;
  for (int i = 0; i < n_layers; ++i) {
    const size_t b = mofq_workspace_bytes(&w[i], nullptr, n_candidates, MOFQ_ERR_TENSOR, w_cfg);
    if (!b) return 0;
    total += b;
  }
  return total;
}

int mofq_select_layers(int32_t n_layers, const mofq_tensor_t* w, const int32_t* candidates,
                       int32_t n_candidates, const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out,
                       mofq_result_t* results, void* ws, size_t ws_bytes, void* stream,
                       void* side_stream) {
  return mofq_select_layers_timed(n_layers, w, candidates, n_candidates, w_cfg, w_out, results, ws,
                                  ws_bytes, stream, side_stream, nullptr, nullptr);
}

int mofq_select_layers_timed(int32_t n_layers, const mofq_tensor_t* w, const int32_t* candidates,
                             int32_t n_candidates, const mofq_scale_cfg_t* w_cfg,
                             const mofq_qout_t* w_out, mofq_result_t* results, void* ws,
                             size_t ws_bytes, void* stream, void* side_stream,
                             void* const* ev_begin, void* const* ev_end) {
  if (n_layers < 1 || !w || !w_out || !results) return MOFQ_ERR_INVALID_ARG;
  int rc = check_candidates(candidates, n_candidates);
  if (rc) return rc;
  // everything is validated before anything is enqueued
  for (int i = 0; i < n_layers; ++i) {
    if ((rc = check_tensor(&w[i]))) return rc;
    if ((rc = check_cfg(&w[i], w_cfg))) return rc;
    if ((rc = check_out(&w_out[i], true))) return rc;
  }
  const size_t need = mofq_select_layers_workspace_bytes(n_layers, w, n_candidates, w_cfg);
  if (!ws || !need || ws_bytes < need || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // With a second stream the memory-bound tail of a batch (select, code emission) runs beside
  // the ALU-bound searches of the next batch.
  SideWork sw(st, side_stream);
  if ((rc = sw.init())) return rc;
  hipStream_t st2 = sw.side;
  auto join = [&](int status) { return sw.join(status); };
  // Beside the searches the emission has their whole duration to move its bytes: two
  // workgroups per compute unit leave the wave slots to the searches and still finish in time
  // (measured on 256 compute units: 7B-shaped set 15.5 ms per pass against 15.7 with one per
  // compute unit and 18.7 with fewer; 65B-shaped set 123.5 against 140.4 ms, where one per compute
  // unit no longer keeps up with the searches; three to eight per compute unit are no faster).
  const int cus = compute_units();
  int emit_cap = sw.two ? 2 * cus : 0;

  auto emit_params = [&](int i, const WOnlyWs& s) {
    EmitParams e{};
    e.w = w[i].data;
    e.dtype = w[i].dtype;
    e.rows = w[i].rows;
    e.cols = w[i].cols;
    e.ld = w[i].ld;
    e.gran = w_cfg->gran;
    e.group = w_cfg->group_size;
    e.scale_f16_out = w_cfg->scale_dtype == MOFQ_F16;
    e.n_cand = n_candidates;
    for (int c = 0; c < n_candidates; ++c) {
      e.fmt[c] = candidates[c];
      e.scale[c] = s.scale[c];
      e.clip[c] = s.clip[c];
      e.err[c] = s.err[c];
    }
    e.result = &results[i];
    e.out = w_out[i];
    e.max_blocks = emit_cap;
    return e;
  };

  char* base = static_cast<char*>(ws);
  for (int i0 = 0, nb = 0; i0 < n_layers; i0 += nb) {
    nb = batch_length(n_layers, w, i0, cus);
    WOnlyWs slot[kFinishBatch];
    FinishParams fin[kFinishBatch];
    DecideParams big[kFinishBatch];
    int n_fin = 0, fin_of[kFinishBatch], n_big = 0, big_of[kFinishBatch];
    // 1. the searches, back to back; the tensors of one row length share a launch
    for (int j = 0; j < nb; ++j) {
      const int64_t units = mofq_num_units(w[i0 + j].rows, w[i0 + j].cols, w_cfg->gran, w_cfg->group_size);
      slot[j] = carve_w_only(base, units, n_candidates, w_cfg->gran, w_cfg->n_clip);
      base += slot[j].bytes;
    }
    int first[kFinishBatch];
    plan_search_groups(w + i0, nb, candidates, n_candidates, first);
    const bool one_launch = one_sweep_launch(candidates, n_candidates);
    for (int j = 0; j < nb; ++j) {
      if (first[j] != j) continue;
      // A launch over several tensors exists only where the whole candidate list is one
      // launch (plan_search_groups joins nothing otherwise); longer lists go tensor by tensor
      // through sweep_candidates, which splits them into launches of at most two formats.
      SweepParams sp[kSweepGroupMax];
      int g = 0, last = j;
      for (int k = j; k < nb; ++k)
        if (first[k] == j) {
          if (one_launch && (rc = sweep_params(&w[i0 + k], candidates, 0, n_candidates, w_cfg, slot[k], &sp[g])))
            return join(rc);
          ++g;
          last = k;
        }
      if (ev_begin && hipEventRecord(static_cast<hipEvent_t>(ev_begin[i0 + j]), st) != hipSuccess) return join(MOFQ_ERR_HIP);
      if (g > 1) {
        if (!one_launch) return join(MOFQ_ERR_INVALID_ARG);   // cannot happen: see plan_search_groups
        if ((rc = launch_sweep_group(sp, g, st))) return join(rc);
      } else {
        if ((rc = sweep_candidates(&w[i0 + j], candidates, n_candidates, w_cfg, slot[j], st))) return join(rc);
      }
      if (ev_end && hipEventRecord(static_cast<hipEvent_t>(ev_end[i0 + last]), st) != hipSuccess) return join(MOFQ_ERR_HIP);
    }
    for (int j = 0; j < nb; ++j) {
      const int i = i0 + j;
      const int64_t units = mofq_num_units(w[i].rows, w[i].cols, w_cfg->gran, w_cfg->group_size);
      DecideParams d{};
      d.units = units;
      d.n_cand = n_candidates;
      for (int c = 0; c < n_candidates; ++c) d.err[c] = slot[j].err[c];
      d.energy = slot[j].energy;
      d.part = slot[j].decide_part;
      d.result = &results[i];
      if (units <= kFinishMaxUnits) {
        FinishParams& f = fin[n_fin];
        f = FinishParams{};
        f.d = d;
        f.scale_f16_out = w_cfg->scale_dtype == MOFQ_F16;
        for (int c = 0; c < n_candidates; ++c) { f.scale[c] = slot[j].scale[c]; f.clip[c] = slot[j].clip[c]; }
        f.out_scales = w_out[i].scales;
        f.out_clip = w_out[i].clip_idx;
        f.out_unit_err = w_out[i].unit_err;
        fin_of[n_fin++] = j;
      } else {
        // many units (group-wise scales): the two-stage reduce and the per-unit kernel of the
        // single-tensor path, after the batch's searches
        big[n_big] = d;
        big_of[n_big++] = j;
      }
    }
    if (i0 + nb >= n_layers) emit_cap = 0;   // nothing runs beside the last batch's emission
    // 2. on the second stream, once the batch's searches are done: reduce + select + per-unit
    //    outputs of the batch in one launch, then the codes of the winners.  The next batch's
    //    searches follow on the caller's stream meanwhile; every tensor has its own workspace.
    if ((rc = sw.fork())) return join(rc);
    if (n_fin && (rc = launch_finish_batch(fin, n_fin, st2))) return join(rc);
    for (int q = 0; q < n_fin; ++q) {
      const int j = fin_of[q];
      EmitParams e = emit_params(i0 + j, slot[j]);
      e.out.scales = nullptr;
      e.out.clip_idx = nullptr;
      e.out.unit_err = nullptr;
      if ((rc = launch_emit(e, st2))) return join(rc);
    }
    for (int q = 0; q < n_big; ++q) {
      if ((rc = launch_decide(big[q], st2))) return join(rc);
      if ((rc = launch_emit(emit_params(i0 + big_of[q], slot[big_of[q]]), st2))) return join(rc);
    }
  }
  return join(MOFQ_OK);
}

int mofq_calibrate_absmax(const mofq_tensor_t* x, float* absmax, void* ws, size_t ws_bytes,
                          void* stream) {
  int rc = check_tensor(x);
  if (rc) return rc;
  if (!absmax) return MOFQ_ERR_INVALID_ARG;
  const mofq_scale_cfg_t cfg = x_cfg();
  if ((rc = check_cfg(x, &cfg))) return rc;
  const WOnlyWs s = carve_w_only(ws, 1, 1, MOFQ_PER_TENSOR, 1);
  if (!ws || ws_bytes < s.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  SweepParams p{};
  p.w = x->data;
  p.dtype = x->dtype;
  p.rows = x->rows;
  p.cols = x->cols;
  p.ld = x->ld;
  p.absmax_part = s.absmax_part;
  p.energy_part = s.energy_part;
  return launch_running_absmax(p, absmax, static_cast<hipStream_t>(stream));
}

int mofq_select_calibrated(const mofq_tensor_t* x, const int32_t* candidates, int32_t n_candidates,
                           const float* absmax, const mofq_qout_t* x_out, mofq_result_t* result,
                           void* ws, size_t ws_bytes, void* stream) {
  int rc = check_tensor(x);
  if (rc) return rc;
  if ((rc = check_candidates(candidates, n_candidates))) return rc;
  if (x_out && (rc = check_out(x_out, true))) return rc;
  if (!absmax || !result) return MOFQ_ERR_INVALID_ARG;
  const mofq_scale_cfg_t cfg = x_cfg();   // per-tensor, ratio 1, fp32 scale
  if ((rc = check_cfg(x, &cfg))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const WOnlyWs s = carve_w_only(ws, 1, n_candidates, MOFQ_PER_TENSOR, 1);
  if (!ws || ws_bytes < s.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  if ((rc = sweep_candidates(x, candidates, n_candidates, &cfg, s, st, absmax))) return rc;
  DecideParams d{};
  d.units = 1;
  d.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) d.err[c] = s.err[c];
  d.energy = s.energy;
  d.result = result;
  if ((rc = launch_decide(d, st))) return rc;
  if (!x_out) return MOFQ_OK;
  EmitParams e{};
  e.w = x->data;
  e.dtype = x->dtype;
  e.rows = x->rows;
  e.cols = x->cols;
  e.ld = x->ld;
  e.gran = MOFQ_PER_TENSOR;
  e.group = 0;
  e.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) {
    e.fmt[c] = candidates[c];
    e.scale[c] = s.scale[c];
    e.clip[c] = s.clip[c];
    e.err[c] = s.err[c];
  }
  e.result = result;
  e.out = *x_out;
  return launch_emit(e, st);
}

size_t mofq_select_units_workspace_bytes(const mofq_tensor_t* w, int32_t n_candidates,
                                         const mofq_scale_cfg_t* w_cfg) {
  const size_t base = mofq_workspace_bytes(w, nullptr, n_candidates, MOFQ_ERR_TENSOR, w_cfg);
  if (!base || w_cfg->gran == MOFQ_PER_TENSOR) return 0;
  const int64_t units = mofq_num_units(w->rows, w->cols, w_cfg->gran, w_cfg->group_size);
  return base + (static_cast<size_t>(units) * sizeof(double) + kAlign - 1) / kAlign * kAlign;
}

int mofq_select_units(const mofq_tensor_t* w, const int32_t* candidates, int32_t n_candidates,
                      const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out, uint8_t* unit_format,
                      mofq_result_t* result, double* mixed_err, void* ws, size_t ws_bytes,
                      void* stream) {
  int rc = check_tensor(w);
  if (rc) return rc;
  if ((rc = check_cfg(w, w_cfg))) return rc;
  if ((rc = check_candidates(candidates, n_candidates))) return rc;
  if ((rc = check_out(w_out, true))) return rc;
  if (!result || !unit_format || !mixed_err) return MOFQ_ERR_INVALID_ARG;
  if (w_cfg->gran == MOFQ_PER_TENSOR) return MOFQ_ERR_UNSUPPORTED;   // that unit is the layer: mofq_select_layer
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t units = mofq_num_units(w->rows, w->cols, w_cfg->gran, w_cfg->group_size);
  const WOnlyWs s = carve_w_only(ws, units, n_candidates, w_cfg->gran, w_cfg->n_clip);
  const size_t need = mofq_select_units_workspace_bytes(w, n_candidates, w_cfg);
  if (!ws || !need || ws_bytes < need || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  double* picked = reinterpret_cast<double*>(static_cast<char*>(ws) + s.bytes);
  if ((rc = sweep_candidates(w, candidates, n_candidates, w_cfg, s, st))) return rc;
  // the layer-wise view, as mofq_select_layer reports it
  DecideParams d{};
  d.units = units;
  d.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) d.err[c] = s.err[c];
  d.energy = s.energy;
  d.part = s.decide_part;
  d.result = result;
  if ((rc = launch_decide(d, st))) return rc;
  // per unit
  PickUnitsParams pk{};
  pk.units = units;
  pk.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) pk.err[c] = s.err[c];
  pk.unit_fmt = unit_format;
  pk.picked_err = picked;
  if ((rc = launch_pick_units(pk, st))) return rc;
  DecideParams m{};
  m.units = units;
  m.n_cand = 1;
  m.err[0] = picked;
  m.part = s.decide_part;
  m.tensor_err_out = mixed_err;
  if ((rc = launch_decide(m, st))) return rc;
  EmitParams e{};
  e.w = w->data;
  e.dtype = w->dtype;
  e.rows = w->rows;
  e.cols = w->cols;
  e.ld = w->ld;
  e.gran = w_cfg->gran;
  e.group = w_cfg->group_size;
  e.scale_f16_out = w_cfg->scale_dtype == MOFQ_F16;
  e.n_cand = n_candidates;
  for (int c = 0; c < n_candidates; ++c) {
    e.fmt[c] = candidates[c];
    e.scale[c] = s.scale[c];
    e.clip[c] = s.clip[c];
    e.err[c] = s.err[c];
  }
  e.result = nullptr;
  e.unit_fmt = unit_format;
  e.out = *w_out;
  return launch_emit(e, st);
}

int mofq_select_layer(const mofq_tensor_t* w, const mofq_tensor_t* x, const int32_t* candidates,
                      int32_t n_candidates, int32_t metric, const mofq_scale_cfg_t* w_cfg,
                      const mofq_qout_t* w_out, const mofq_qout_t* x_out, mofq_result_t* result,
                      void* ws, size_t ws_bytes, void* stream) {
  return mofq_select_layer_timed(w, x, candidates, n_candidates, metric, w_cfg, w_out, x_out,
                                 result, ws, ws_bytes, stream, nullptr, nullptr);
}

size_t mofq_select_layers_wa_workspace_bytes(int32_t n_layers, const mofq_tensor_t* w, const mofq_tensor_t* x,
                                             int32_t n_candidates, int32_t metric,
                                             const mofq_scale_cfg_t* w_cfg) {
  if (n_layers < 1 || !w || !x || !w_cfg) return 0;
  if (metric != MOFQ_ERR_LAYER_OUTPUT && metric != MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT) return 0;
  size_t need = 0;
  for (int i = 0; i < n_layers; ++i) {
    const size_t b = mofq_workspace_bytes(&w[i], &x[i], n_candidates, metric, w_cfg);
    if (!b) return 0;
    need = std::max(need, b);
  }
  if (n_candidates == 2 && w_cfg->gran == MOFQ_PER_TENSOR)
    need = std::max(need, wa_fused_bytes(n_layers, w, x, metric == MOFQ_ERR_LAYER_OUTPUT));
  return need;
}

int mofq_select_layers_wa_timed(int32_t n_layers, const mofq_tensor_t* w, const mofq_tensor_t* x,
                                const int32_t* candidates, int32_t n_candidates, int32_t metric,
                                const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out,
                                const mofq_qout_t* x_out, mofq_result_t* results, void* ws,
                                size_t ws_bytes, void* stream, void* const* ev_begin, void* const* ev_end) {
  if (n_layers < 1 || !w || !x || !w_out || !results) return MOFQ_ERR_INVALID_ARG;
  if (metric != MOFQ_ERR_LAYER_OUTPUT && metric != MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT) return MOFQ_ERR_INVALID_ARG;
  int rc = check_candidates(candidates, n_candidates);
  if (rc) return rc;
  // everything is validated before anything is enqueued
  for (int i = 0; i < n_layers; ++i) {
    if ((rc = check_tensor(&w[i]))) return rc;
    if ((rc = check_cfg(&w[i], w_cfg))) return rc;
    if ((rc = check_out(&w_out[i], true))) return rc;
    if ((rc = check_wa(&w[i], &x[i], candidates, n_candidates, w_cfg))) return rc;
    if (x_out && (rc = check_out(&x_out[i], true))) return rc;
  }
  const size_t need = mofq_select_layers_wa_workspace_bytes(n_layers, w, x, n_candidates, metric, w_cfg);
  if (!ws || !need || ws_bytes < need || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
  return select_layers_wa(n_layers, w, x, candidates, n_candidates, metric, w_cfg, w_out, x_out, results, ws,
                          ws_bytes, static_cast<hipStream_t>(stream), ev_begin, ev_end);
}

int mofq_select_layers_wa(int32_t n_layers, const mofq_tensor_t* w, const mofq_tensor_t* x,
                          const int32_t* candidates, int32_t n_candidates, int32_t metric,
                          const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out, const mofq_qout_t* x_out,
                          mofq_result_t* results, void* ws, size_t ws_bytes, void* stream) {
  return mofq_select_layers_wa_timed(n_layers, w, x, candidates, n_candidates, metric, w_cfg, w_out, x_out,
                                     results, ws, ws_bytes, stream, nullptr, nullptr);
}

int mofq_select_layer_static(const mofq_tensor_t* w, const int32_t* candidates, int32_t n_candidates,
                             const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out,
                             mofq_result_t* result, void* stream) {
  int rc = check_tensor(w);
  if (rc) return rc;
  if ((rc = check_cfg(w, w_cfg))) return rc;
  if ((rc = check_candidates(candidates, n_candidates))) return rc;
  if ((rc = check_out(w_out, true))) return rc;
  if (!result) return MOFQ_ERR_INVALID_ARG;
  const size_t need = mofq_workspace_bytes(w, nullptr, n_candidates, MOFQ_ERR_TENSOR, w_cfg);
  if (!need || need > MOFQ_STATIC_WORKSPACE_BYTES) return MOFQ_ERR_WORKSPACE;   // beyond the built-in array
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  return select_w_only(w, candidates, n_candidates, w_cfg, w_out, result, ws, MOFQ_STATIC_WORKSPACE_BYTES,
                       static_cast<hipStream_t>(stream), nullptr, nullptr);
}

int mofq_select_layer_timed(const mofq_tensor_t* w, const mofq_tensor_t* x,
                            const int32_t* candidates, int32_t n_candidates, int32_t metric,
                            const mofq_scale_cfg_t* w_cfg, const mofq_qout_t* w_out,
                            const mofq_qout_t* x_out, mofq_result_t* result, void* ws,
                            size_t ws_bytes, void* stream, void* ev_score_begin,
                            void* ev_score_end) {
  hipEvent_t ev0 = static_cast<hipEvent_t>(ev_score_begin);
  hipEvent_t ev1 = static_cast<hipEvent_t>(ev_score_end);
  int rc = check_tensor(w);
  if (rc) return rc;
  if ((rc = check_cfg(w, w_cfg))) return rc;
  if ((rc = check_candidates(candidates, n_candidates))) return rc;
  if ((rc = check_out(w_out, true))) return rc;
  if (!result) return MOFQ_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!x) {
    if (metric != MOFQ_ERR_TENSOR) return MOFQ_ERR_INVALID_ARG;
    (void)x_out;
    return select_w_only(w, candidates, n_candidates, w_cfg, w_out, result, ws, ws_bytes, st, ev0, ev1);
  }
  if (metric == MOFQ_ERR_LAYER_OUTPUT_W_ONLY) {
    if ((rc = check_wo_output(w, x, candidates, n_candidates, w_cfg))) return rc;
    const WoOutWs a = carve_wo_output(ws, w, x, n_candidates, w_cfg);
    if (!ws || ws_bytes < a.bytes || !aligned16(ws)) return MOFQ_ERR_WORKSPACE;
    if ((rc = wo_output_score(w, x, candidates, n_candidates, w_cfg, a, st, ev0, ev1))) return rc;
    DecideParams d{};
    d.units = a.blocks;
    d.n_cand = n_candidates;
    for (int c = 0; c < n_candidates; ++c) d.err[c] = a.part[c];
    d.energy = a.part[2];
    d.result = result;
    if ((rc = launch_decide(d, st))) return rc;
    // second quantize_layer call of Algorithm 1: W in the chosen format
    EmitParams e{};
    e.w = w->data;
    e.dtype = w->dtype;
    e.rows = w->rows;
    e.cols = w->cols;
    e.ld = w->ld;
    e.gran = w_cfg->gran;
    e.group = 0;
    e.scale_f16_out = w_cfg->scale_dtype == MOFQ_F16;
    e.n_cand = n_candidates;
    for (int c = 0; c < n_candidates; ++c) {
      e.fmt[c] = candidates[c];
      e.scale[c] = a.wrec.scale[c];
      e.clip[c] = a.wrec.clip[c];
      e.err[c] = a.wrec.err[c];
    }
    e.result = result;
    e.out = *w_out;
    return launch_emit(e, st);
  }
  if (metric != MOFQ_ERR_LAYER_OUTPUT && metric != MOFQ_ERR_LAYER_OUTPUT_FP8_UNIT)
    return MOFQ_ERR_INVALID_ARG;
  if ((rc = check_wa(w, x, candidates, n_candidates, w_cfg))) return rc;
  if (x_out && (rc = check_out(x_out, true))) return rc;
  return select_layers_wa(1, w, x, candidates, n_candidates, metric, w_cfg, w_out, x_out, result, ws, ws_bytes,
                          st, ev_score_begin ? &ev_score_begin : nullptr,
                          ev_score_end ? &ev_score_end : nullptr);
}

}  // extern "C"
