// C ABI of the RAD library (see include/rad.h): argument checking, store and
// workspace management, and the launch sequences of the entry points.  All
// arithmetic of the method happens in the kernels this file launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <utility>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/rad.h"
#include "kernels.hpp"

using namespace rad;

// --------------------------------------------------------------------- ctx
struct rad_ctx {
  hipStream_t stream = nullptr;
  int device = 0;
  std::string err;
  int key_shift = 0;
  // side stream of the recurrent model's backward pass (created on first use): the gradients formed per chunk of
  // time steps run there, beside the chain of dX GEMMs
  hipStream_t side = nullptr;
  hipEvent_t ev_ready[2] = {nullptr, nullptr}, ev_done[2] = {nullptr, nullptr}, ev_join = nullptr;
  // timing
  bool timing = false;
  std::string filter;
  struct Rec { std::string name; hipEvent_t a, b; double alg_flops, exe_flops; };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  // grow-only workspaces
  void* ws[11] = {};
  size_t ws_bytes[11] = {};
  float* loss_dev = nullptr;
};

enum { WS_BITMAP = 0, WS_DENSE = 1, WS_ROWLOSS = 2, WS_COLSUM = 3, WS_SPLITK = 4, WS_WT = 5, WS_PROJ_R = 6, WS_PROJ_T = 7,
       WS_PROJ_TB = 8, WS_REINDEX = 9, WS_CONVG = 10 };

static const char* kNoCtx = "no context";

// Keep bitmap of rad_sample_pack_static: device memory this library owns from load to exit on every GPU it runs
// on, so that the call has nothing to allocate.  The name `scratch` is the host-side stand-in of the symbol, not
// a device address: host code uses the address hipGetSymbolAddress returns for the current device, kept per
// device in g_scratch (each GPU holds a copy of the array at an address of its own).
constexpr size_t kScratchWords = RAD_STATIC_SCRATCH_BYTES / 4;
static __device__ __align__(256) uint32_t scratch[kScratchWords];
constexpr int kMaxDevices = 64;
static uint32_t* g_scratch[kMaxDevices] = {};

// with `device` current: the device address of `scratch` on it (looked up once per device)
static hipError_t scratch_resolve(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch[device]) return hipSuccess;
  void* ptr = nullptr;
  hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!ptr) return hipErrorInvalidSymbol;
  g_scratch[device] = static_cast<uint32_t*>(ptr);
  return hipSuccess;
}

static rad_status fail(rad_ctx* c, rad_status s, const std::string& msg) {
  if (c) c->err = msg;
  return s;
}
static rad_status hip_fail(rad_ctx* c, hipError_t e, const char* what) {
  return fail(c, RAD_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(ctx, expr)                                        \
  do {                                                            \
    hipError_t e__ = (expr);                                      \
    if (e__ != hipSuccess) return hip_fail(ctx, e__, #expr);      \
  } while (0)
#define RAD_TRY(expr)                                             \
  do {                                                            \
    rad_status s__ = (expr);                                      \
    if (s__ != RAD_OK) return s__;                                \
  } while (0)

static rad_status ws_get(rad_ctx* c, int which, size_t bytes, void** out) {
  if (bytes > c->ws_bytes[which]) {
    if (c->ws[which]) {
      // either stream may still read the old buffer (the recurrent model's backward pass swaps the two)
      HIP_TRY(c, hipStreamSynchronize(c->stream));
      if (c->side) HIP_TRY(c, hipStreamSynchronize(c->side));
      HIP_TRY(c, hipFree(c->ws[which]));
      c->ws[which] = nullptr; c->ws_bytes[which] = 0;
    }
    HIP_TRY(c, hipMalloc(&c->ws[which], bytes));
    c->ws_bytes[which] = bytes;
  }
  *out = c->ws[which];
  return RAD_OK;
}

// runs `launch` (which enqueues exactly one logical kernel and reports its
// label through *name), bracketed by events when timing is on
template <class F>
static hipError_t timed(rad_ctx* c, const char* name, F launch) {
  const char* nm = name;
  if (!c->timing || (!c->filter.empty() && std::string(name).find(c->filter) == std::string::npos))
    return launch(&nm);
  hipEvent_t a, b;
  for (hipEvent_t* ev : {&a, &b}) {
    if (!c->pool.empty()) { *ev = c->pool.back(); c->pool.pop_back(); }
    else { hipError_t e = hipEventCreate(ev); if (e != hipSuccess) return e; }
  }
  hipError_t e = hipEventRecord(a, c->stream);
  if (e != hipSuccess) return e;
  e = launch(&nm);
  if (e != hipSuccess) return e;
  e = hipEventRecord(b, c->stream);
  if (e != hipSuccess) return e;
  c->recs.push_back({nm, a, b, 0.0, 0.0});
  return hipSuccess;
}

extern "C" int64_t rad_fixed_k(double p, int64_t d) {
  int64_t k = (int64_t)std::ceil(p * (double)d - 1e-9);
  if (k < 1) k = 1;
  if (k > d) k = d;
  return k;
}

extern "C" rad_status rad_ctx_create(rad_ctx** out, void* hip_stream) {
  if (!out) return RAD_ERR_NULL;
  *out = nullptr;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || n < 1) return RAD_ERR_DEVICE;
  rad_ctx* c = new rad_ctx();
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (hipGetDevice(&c->device) != hipSuccess) { delete c; return RAD_ERR_DEVICE; }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, c->device) != hipSuccess) { delete c; return RAD_ERR_DEVICE; }
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) { delete c; return RAD_ERR_UNSUPPORTED; }
  if (hipMalloc(reinterpret_cast<void**>(&c->loss_dev), sizeof(float)) != hipSuccess) { delete c; return RAD_ERR_DEVICE; }
  if (scratch_resolve(c->device) != hipSuccess) { (void)hipFree(c->loss_dev); delete c; return RAD_ERR_DEVICE; }
  *out = c;
  return RAD_OK;
}

extern "C" rad_status rad_ctx_destroy(rad_ctx* c) {
  if (!c) return RAD_ERR_NULL;
  (void)hipStreamSynchronize(c->stream);
  for (auto& r : c->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
  for (hipEvent_t e : {c->ev_ready[0], c->ev_ready[1], c->ev_done[0], c->ev_done[1], c->ev_join}) if (e) (void)hipEventDestroy(e);
  for (auto& e : c->pool) (void)hipEventDestroy(e);
  for (void* w : c->ws) if (w) (void)hipFree(w);
  if (c->loss_dev) (void)hipFree(c->loss_dev);
  delete c;
  return RAD_OK;
}

extern "C" const char* rad_last_error(const rad_ctx* c) { return c ? c->err.c_str() : kNoCtx; }

extern "C" rad_status rad_ctx_synchronize(rad_ctx* c) {
  if (!c) return RAD_ERR_NULL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return RAD_OK;
}

extern "C" rad_status rad_ctx_timing(rad_ctx* c, const char* filter) {
  if (!c) return RAD_ERR_NULL;
  if (filter && filter[0] == '\0') { c->timing = false; return RAD_OK; }
  c->timing = true;
  c->filter = filter ? filter : "";
  return RAD_OK;
}

extern "C" rad_status rad_ctx_timing_reset(rad_ctx* c) {
  if (!c) return RAD_ERR_NULL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (auto& r : c->recs) { c->pool.push_back(r.a); c->pool.push_back(r.b); }
  c->recs.clear();
  return RAD_OK;
}

extern "C" rad_status rad_ctx_timing_read(rad_ctx* c, const char* name, int64_t* launches, double* total_ms) {
  if (!c || !launches || !total_ms) return RAD_ERR_NULL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  int64_t n = 0; double ms = 0.0;
  for (auto& r : c->recs) {
    if (name && r.name.find(name) == std::string::npos) continue;
    float t = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&t, r.a, r.b));
    ms += t; ++n;
  }
  *launches = n; *total_ms = ms;
  return RAD_OK;
}

extern "C" rad_status rad_ctx_timing_read_flops(rad_ctx* c, const char* name, double* algorithmic, double* executed) {
  if (!c || !algorithmic || !executed) return RAD_ERR_NULL;
  double a = 0.0, x = 0.0;
  for (auto& r : c->recs) {
    if (name && r.name.find(name) == std::string::npos) continue;
    a += r.alg_flops; x += r.exe_flops;
  }
  *algorithmic = a; *executed = x;
  return RAD_OK;
}

// test hook: the keys of the next draw (one store_plan) are shifted right by `shift` bits before selection,
// which makes equal keys frequent and so exercises the tie rule of the fixed-k draw; the draw resets it
extern "C" rad_status rad_debug_key_shift(rad_ctx* c, int32_t shift) {
  if (!c) return RAD_ERR_NULL;
  if (shift < 0 || shift > 31) return fail(c, RAD_ERR_PARAM, "key shift must be in [0, 31]");
  c->key_shift = shift;
  return RAD_OK;
}

// measured ceilings: `reps` launches of one probe kernel between two events on the context's stream
extern "C" rad_status rad_probe_ceiling(rad_ctx* c, int32_t kind, const void* operands, void* sink, uint64_t bytes,
                                        int32_t reps, double* units_per_s) {
  if (!c) return RAD_ERR_NULL;
  if (!operands || !sink || !units_per_s) return fail(c, RAD_ERR_NULL, "null argument");
  if (kind < 0 || kind > 5) return fail(c, RAD_ERR_PARAM, "unknown probe kind");
  if (reps < 1 || reps > 10000) return fail(c, RAD_ERR_PARAM, "reps must be in [1, 10000]");
  if (bytes < probe_min_bytes(kind) || bytes % 16 != 0 || bytes > (uint64_t(1) << 36))
    return fail(c, RAD_ERR_SHAPE, "operand buffer too small for this probe, not a multiple of 16 bytes, or above 64 GiB");
  if ((reinterpret_cast<uintptr_t>(operands) | reinterpret_cast<uintptr_t>(sink)) & 15)
    return fail(c, RAD_ERR_PARAM, "buffers must be 16-byte aligned");
  const int iters = 128;                 // MFMA loops: 128 iterations = the flops of one 4096^3 GEMM over the chip
  hipEvent_t e0, e1;
  HIP_TRY(c, hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(c, RAD_ERR_DEVICE, "event"); }
  hipError_t e = hipSuccess;
  for (int w = 0; w < 3 && e == hipSuccess; ++w) e = launch_probe(kind, operands, sink, bytes, iters, c->stream);
  if (e == hipSuccess) e = hipEventRecord(e0, c->stream);
  for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch_probe(kind, operands, sink, bytes, iters, c->stream);
  if (e == hipSuccess) e = hipEventRecord(e1, c->stream);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (e != hipSuccess) return hip_fail(c, e, "ceiling probe");
  *units_per_s = probe_units(kind, bytes, iters) * reps / ((double)ms * 1e-3);
  return RAD_OK;
}

// ------------------------------------------------------------------- store
struct rad_store {
  int scheme = 0, dtype = 0;
  int rows = 0, cols = 0, d_out = 0, steps = 1;
  int k = 0;
  int k_pitch = 0;                // shared scheme: row pitch of the compact values, k rounded up to 8 (padding stays zero)
  double p = 1.0;
  float scale = 1.f;
  int64_t capacity = 0;
  void* values = nullptr;
  uint16_t* indices = nullptr;
  uint32_t* row_ptr = nullptr;
  uint16_t* bucket_off = nullptr;
  uint32_t* row_cnt = nullptr;
  bool index_free = false;        // keep values only; columns are drawn again before the backward pass
  rad_sampling last_plan{};       // sampling parameters of the last plan (what an index-free store is rebuilt from)
  bool planned = false;
  uint64_t proj_seed = 0;         // projection scheme: the sampling parameters of the last forward, from which the
  uint32_t proj_stream = 0, proj_step = 0;   //   backward pass regenerates R
  bool proj_valid = false;
  uint16_t* mult = nullptr;       // with-replacement draws: draw counts, [steps * plan rows][k] in entry order
  uint32_t* bits = nullptr;
  uint32_t* bitmap = nullptr;     // transient, points into a context workspace after a plan
  int* overflow = nullptr;        // sticky flag: a Bernoulli draw exceeded the capacity (stays set until read)
  int* max_seg = nullptr;         // longest (row, bucket) segment of the last plan
  bool flags_external = false;    // both live in the owning model's flag array
  int bits_pitch = 0, nb = 0, bm_pitch = 0;
  int plan_rows_per_step = 0;     // rows (per example / Bernoulli), 1 (shared), 0 (exact)
  size_t elem() const { return dtype == kBF16 ? 2 : 4; }
  // bf16 stores with per-entry draws keep (value, column) in one 32-bit entry
  bool per_entry() const { return scheme == kBernoulli || scheme == kFixedKPerExample || replace(); }
  bool paired() const { return dtype == kBF16 && per_entry() && !index_free; }
  bool replace() const { return scheme == kReplaceShared || scheme == kReplacePerExample; }
  bool project() const { return scheme == kProjectShared || scheme == kProjectPerExample; }
  bool compact() const { return scheme == kFixedKShared || project(); }   // values are [rows][k_pitch]
  // rows hold a number of entries that only the plan kernel knows
  bool counted_rows() const { return scheme == kBernoulli || replace(); }
  size_t bitmap_words() const { return (size_t)steps * plan_rows_per_step * bm_pitch; }
};

static StoreView store_view(const rad_store* s, int slot) {
  StoreView v;
  v.values = s->values;
  v.capacity = s->capacity;
  v.rows = s->rows; v.cols = s->cols; v.nb = s->nb; v.bm_pitch = s->bm_pitch;
  v.scale = s->scale;
  v.plan_row_stride = (s->scheme == kFixedKShared || s->scheme == kReplaceShared) ? 0 : 1;
  v.idx_shared = s->scheme == kFixedKShared ? 1 : 0;
  v.paired = s->paired() ? 1 : 0;
  v.may_overflow = s->scheme == kBernoulli ? 1 : 0;
  v.indices = s->scheme == kFixedKShared ? s->indices + (size_t)slot * s->k : s->indices;
  v.shared_k = s->scheme == kFixedKShared ? s->k : 0;
  v.mult = s->mult ? s->mult + (size_t)slot * s->plan_rows_per_step * s->k : nullptr;
  v.mult_pitch = s->k;
  v.row_ptr = s->row_ptr ? s->row_ptr + (size_t)slot * s->rows : nullptr;
  const size_t prow0 = (size_t)slot * s->plan_rows_per_step;
  v.bucket_off = s->bucket_off ? s->bucket_off + prow0 * (s->nb + 1) : nullptr;
  v.bitmap = s->bitmap ? s->bitmap + prow0 * s->bm_pitch : nullptr;
  return v;
}

static rad_status check_layer(rad_ctx* c, const rad_layer* L) {
  if (!L) return fail(c, RAD_ERR_NULL, "layer is null");
  if (L->dtype != RAD_F32 && L->dtype != RAD_BF16) return fail(c, RAD_ERR_PARAM, "unknown dtype");
  if (L->kind != RAD_LINEAR && L->kind != RAD_CONV2D) return fail(c, RAD_ERR_PARAM, "unknown layer kind");
  if (L->batch < 1 || L->d_in < 1 || L->d_out < 1) return fail(c, RAD_ERR_SHAPE, "batch, d_in and d_out must be positive");
  if (L->batch > (1 << 24) || L->d_in > (1 << 24) || L->d_out > (1 << 24))
    return fail(c, RAD_ERR_SHAPE, "dimension above 2^24");
  if (L->kind == RAD_CONV2D) {
    if (L->c_in < 1 || L->c_out < 1 || L->h < 1 || L->w < 1 || L->kh < 1 || L->kw < 1)
      return fail(c, RAD_ERR_SHAPE, "conv dimensions must be positive");
    if (2 * L->pad != L->kh - 1 || 2 * L->pad != L->kw - 1) return fail(c, RAD_ERR_SHAPE, "conv must keep the spatial size");
    if ((int64_t)L->c_in * L->h * L->w != L->d_in || (int64_t)L->c_out * L->h * L->w != L->d_out)
      return fail(c, RAD_ERR_SHAPE, "d_in/d_out do not match the conv shape");
    if (L->dtype != RAD_F32) return fail(c, RAD_ERR_UNSUPPORTED, "conv layers are fp32 only");
  }
  return RAD_OK;
}

static rad_status check_scheme(rad_ctx* c, int scheme, double p) {
  if (scheme < RAD_EXACT || scheme > RAD_PROJECT_PER_EXAMPLE) return fail(c, RAD_ERR_PARAM, "unknown sampling scheme");
  if (!(p > 0.0) || p > 1.0) return fail(c, RAD_ERR_PARAM, "p must be in (0, 1]");
  return RAD_OK;
}

extern "C" rad_status rad_store_destroy(rad_store* s) {
  if (!s) return RAD_ERR_NULL;
  for (void* p : {(void*)s->values, (void*)s->indices, (void*)s->row_ptr, (void*)s->bucket_off, (void*)s->row_cnt, (void*)s->mult,
                  (void*)s->bits, s->flags_external ? nullptr : (void*)s->overflow})
    if (p) (void)hipFree(p);
  delete s;
  return RAD_OK;
}

extern "C" rad_status rad_store_create(rad_ctx* c, const rad_layer* L, int32_t scheme, double p, int32_t steps,
                                       rad_store** out) {
  if (!c) return RAD_ERR_NULL;
  if (!out) return fail(c, RAD_ERR_NULL, "out is null");
  *out = nullptr;
  RAD_TRY(check_layer(c, L));
  RAD_TRY(check_scheme(c, scheme, p));
  if (steps < 1) return fail(c, RAD_ERR_SHAPE, "steps must be >= 1");
  const bool proj = scheme == RAD_PROJECT_SHARED || scheme == RAD_PROJECT_PER_EXAMPLE;
  if (proj && L->kind != RAD_LINEAR)
    return fail(c, RAD_ERR_UNSUPPORTED, "the projection schemes serve linear layers only");
  if (scheme == RAD_PROJECT_PER_EXAMPLE && rad_fixed_k(p, L->d_in) > 38400)
    return fail(c, RAD_ERR_UNSUPPORTED, "a projection per example keeps at most 38400 numbers per row");
  if (scheme != RAD_EXACT && !proj) {
    if (L->d_in > 65535) return fail(c, RAD_ERR_UNSUPPORTED, "sampled stores need d_in <= 65535 (16-bit indices)");
    if (L->d_in > plan_max_cols(scheme) || (scheme != RAD_BERNOULLI && L->d_in > 16376 && L->d_in % 4 != 0))
      return fail(c, RAD_ERR_UNSUPPORTED, "fixed-k sampling needs d_in <= 16384 (16376 unless a multiple of 4)");
  }
  const double total_rows = (double)steps * (double)L->batch;
  if (total_rows * (double)L->d_in >= 4294967296.0) return fail(c, RAD_ERR_SHAPE, "store above 2^32 entries");
  rad_store* s = new rad_store();
  s->scheme = scheme; s->dtype = L->dtype; s->rows = (int)L->batch; s->cols = (int)L->d_in;
  s->d_out = (int)L->d_out; s->steps = steps; s->p = p;
  s->k = (int)rad_fixed_k(p, L->d_in);
  s->k_pitch = (scheme == RAD_FIXEDK_SHARED || proj) ? (s->k + 7) / 8 * 8 : s->k;
  s->nb = (s->cols + kBucket - 1) / kBucket;
  s->bm_pitch = (s->cols + 31) / 32;
  const int64_t R = (int64_t)steps * s->rows;
  const int64_t n = R * s->cols;
  if (scheme == RAD_EXACT) { s->scale = 1.f; s->capacity = n; s->plan_rows_per_step = 0; }
  else if (scheme == RAD_BERNOULLI) {
    s->scale = (float)(1.0 / p);
    double cap = std::ceil((double)n * p + 8.0 * std::sqrt((double)n * p * (1.0 - p))) + 64.0;
    s->capacity = cap > (double)n ? n : (int64_t)cap;
    s->plan_rows_per_step = s->rows;
  } else if (proj) {
    s->scale = (float)(1.0 / std::sqrt((double)s->k));
    s->capacity = R * s->k_pitch;
    s->plan_rows_per_step = 0;
  } else {
    s->scale = (float)((double)s->cols / (double)s->k);
    s->capacity = R * s->k_pitch;
    s->plan_rows_per_step = (scheme == RAD_FIXEDK_SHARED || scheme == RAD_REPLACE_SHARED) ? 1 : s->rows;
  }
  auto alloc = [&](void** ptr, size_t bytes) -> bool {
    return hipMalloc(ptr, bytes ? bytes : 16) == hipSuccess;
  };
  bool ok = alloc(&s->values, s->paired() ? (size_t)(s->capacity + kPairPad) * 4 : (size_t)s->capacity * s->elem());
  ok = ok && alloc((void**)&s->overflow, 2 * sizeof(int));   // [0] capacity overflow flag, [1] longest bucket segment
  s->max_seg = s->overflow ? s->overflow + 1 : nullptr;
  if (scheme != RAD_EXACT && !proj) {
    const size_t n_idx = scheme == RAD_FIXEDK_SHARED ? (size_t)steps * s->k : (size_t)s->capacity;
    if (!s->paired()) ok = ok && alloc((void**)&s->indices, n_idx * 2);
    ok = ok && alloc((void**)&s->row_ptr, (size_t)(R + 1) * 4);
    ok = ok && alloc((void**)&s->bucket_off, (size_t)steps * s->plan_rows_per_step * (s->nb + 1) * 2);
    if (s->counted_rows()) ok = ok && alloc((void**)&s->row_cnt, (size_t)R * 4);
    if (s->replace()) ok = ok && alloc((void**)&s->mult, (size_t)steps * s->plan_rows_per_step * s->k * 2);
  }
  if (L->relu) {
    s->bits_pitch = (s->d_out + 31) / 32;
    ok = ok && alloc((void**)&s->bits, (size_t)R * s->bits_pitch * 4);
  }
  if (ok) ok = hipMemsetAsync(s->overflow, 0, 2 * sizeof(int), c->stream) == hipSuccess;
  // the padding columns of the compact layout are read by the dW GEMM and never written
  if (ok && scheme == RAD_FIXEDK_SHARED && s->k_pitch != s->k)
    ok = hipMemsetAsync(s->values, 0, (size_t)s->capacity * s->elem(), c->stream) == hipSuccess;
  if (!ok) { rad_store_destroy(s); return fail(c, RAD_ERR_DEVICE, "store allocation failed"); }
  *out = s;
  return RAD_OK;
}

static rad_status store_nnz(rad_ctx* c, const rad_store* s, int64_t* nnz) {
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (s->scheme == RAD_EXACT) { *nnz = s->capacity; return RAD_OK; }
  // shared: k entries per row by construction (the rows of the compact layout may be padded apart)
  if (s->compact()) { *nnz = (int64_t)s->steps * s->rows * s->k; return RAD_OK; }
  uint32_t last = 0;
  HIP_TRY(c, hipMemcpy(&last, s->row_ptr + (size_t)s->steps * s->rows, 4, hipMemcpyDeviceToHost));
  int ov = 0;
  HIP_TRY(c, hipMemcpy(&ov, s->overflow, sizeof(int), hipMemcpyDeviceToHost));
  if (ov) HIP_TRY(c, hipMemset(s->overflow, 0, sizeof(int)));      // reported once
  if (ov || (int64_t)last > s->capacity) return fail(c, RAD_ERR_CAPACITY, "a Bernoulli draw exceeded the store's capacity");
  *nnz = last;
  return RAD_OK;
}

extern "C" rad_status rad_store_get_stats(rad_ctx* c, const rad_store* s, rad_store_stats* out) {
  if (!c) return RAD_ERR_NULL;
  if (!s || !out) return fail(c, RAD_ERR_NULL, "store or out is null");
  int64_t nnz = 0;
  RAD_TRY(store_nnz(c, s, &nnz));
  const int64_t R = (int64_t)s->steps * s->rows;
  out->nnz = (uint64_t)nnz;
  out->value_bytes = (uint64_t)nnz * s->elem();   // entries; the shared scheme's row padding (< 8 per row) is not counted
  out->dense_bytes = (uint64_t)R * s->cols * s->elem();
  out->bit_bytes = s->bits ? (uint64_t)R * s->bits_pitch * 4 : 0;
  if (s->scheme == RAD_EXACT || s->project()) out->index_bytes = 0;
  else if (s->scheme == RAD_FIXEDK_SHARED)
    out->index_bytes = (uint64_t)s->steps * ((uint64_t)s->k * 2 + (uint64_t)(s->nb + 1) * 2);
  else
    out->index_bytes = (s->index_free ? 0 : (uint64_t)nnz * 2) + (uint64_t)R * (s->nb + 1) * 2 +
                       (s->counted_rows() ? (uint64_t)(R + 1) * 4 : 0);
  return RAD_OK;
}

static rad_status backward_view(rad_ctx* c, const rad_store* cs, int slot, StoreView* out);

extern "C" rad_status rad_store_export_csr(rad_ctx* c, const rad_store* s, int64_t* row_ptr, int32_t* col, float* val,
                                           int64_t capacity) {
  if (!c) return RAD_ERR_NULL;
  if (!s || !row_ptr || !col || !val) return fail(c, RAD_ERR_NULL, "null argument");
  int64_t nnz = 0;
  RAD_TRY(store_nnz(c, s, &nnz));
  if (nnz > capacity) return fail(c, RAD_ERR_CAPACITY, "export buffers too small");
  const int64_t R = (int64_t)s->steps * s->rows;
  const bool shared = s->compact();
  // an index-free store is exported from the rebuild the backward pass would read
  const void* vsrc = s->values;
  const uint16_t* isrc = s->indices;
  bool paired = s->paired();
  const bool from_bitmap = s->index_free && s->steps > 1;     // columns are enumerated from the keep bitmap below
  if (from_bitmap && (!s->bitmap || s->dtype != kF32))
    return fail(c, RAD_ERR_PARAM, "the index-free store has no current draw to export");
  if (s->index_free && !from_bitmap) {
    StoreView bv;
    RAD_TRY(backward_view(c, s, 0, &bv));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    vsrc = bv.values; isrc = bv.indices; paired = bv.paired != 0;
  }
  const int64_t n_raw = shared ? R * s->k_pitch : nnz;          // entries held, padding included
  std::vector<unsigned char> vraw((size_t)n_raw * (paired ? 4 : s->elem()));
  if (n_raw) HIP_TRY(c, hipMemcpy(vraw.data(), vsrc, vraw.size(), hipMemcpyDeviceToHost));
  for (int64_t i = 0; i < nnz; ++i) {
    const int64_t src = shared ? (i / s->k) * s->k_pitch + i % s->k : i;
    if (paired) {
      uint32_t u = reinterpret_cast<uint32_t*>(vraw.data())[src] & 0xFFFF0000u;
      std::memcpy(&val[i], &u, 4);
    } else if (s->dtype == kBF16) {
      uint32_t u = (uint32_t)reinterpret_cast<uint16_t*>(vraw.data())[src] << 16;
      std::memcpy(&val[i], &u, 4);
    } else val[i] = reinterpret_cast<float*>(vraw.data())[src];
  }
  if (s->scheme == RAD_EXACT) {
    for (int64_t r = 0; r <= R; ++r) row_ptr[r] = r * s->cols;
    for (int64_t i = 0; i < nnz; ++i) col[i] = (int32_t)(i % s->cols);
    return RAD_OK;
  }
  if (s->project()) {                      // the k numbers of a row are listed as "columns" 0 .. k-1
    for (int64_t r = 0; r <= R; ++r) row_ptr[r] = r * s->k;
    for (int64_t i = 0; i < nnz; ++i) col[i] = (int32_t)(i % s->k);
    return RAD_OK;
  }
  std::vector<uint32_t> rp((size_t)R + 1);
  HIP_TRY(c, hipMemcpy(rp.data(), s->row_ptr, rp.size() * 4, hipMemcpyDeviceToHost));
  for (int64_t r = 0; r <= R; ++r) row_ptr[r] = shared ? r * s->k : (int64_t)rp[(size_t)r];
  if (s->scheme == RAD_FIXEDK_SHARED) {
    std::vector<uint16_t> idx((size_t)s->steps * s->k);
    HIP_TRY(c, hipMemcpy(idx.data(), s->indices, idx.size() * 2, hipMemcpyDeviceToHost));
    for (int64_t r = 0; r < R; ++r)
      for (int j = 0; j < s->k; ++j) col[r * s->k + j] = idx[(size_t)(r / s->rows) * s->k + j];
  } else if (from_bitmap) {
    std::vector<uint32_t> bm(s->bitmap_words());
    HIP_TRY(c, hipMemcpy(bm.data(), s->bitmap, bm.size() * 4, hipMemcpyDeviceToHost));
    for (int64_t r = 0; r < R; ++r) {
      const int64_t prow = s->plan_rows_per_step == s->rows ? r : r / s->rows;
      int64_t e = (int64_t)rp[(size_t)r];
      for (int j = 0; j < s->cols && e < nnz; ++j)
        if ((bm[(size_t)prow * s->bm_pitch + (j >> 5)] >> (j & 31)) & 1u) col[e++] = j;
    }
  } else if (paired) {
    // the bucket of an entry follows from its position in the row
    std::vector<uint16_t> bo((size_t)s->steps * s->plan_rows_per_step * (s->nb + 1));
    HIP_TRY(c, hipMemcpy(bo.data(), s->bucket_off, bo.size() * 2, hipMemcpyDeviceToHost));
    const uint32_t* ent = reinterpret_cast<const uint32_t*>(vraw.data());
    for (int64_t r = 0; r < R; ++r) {
      // one plan row per store row, or per step when every row of the step shares the draw
      const int64_t prow = s->plan_rows_per_step == s->rows ? r : r / s->rows;
      const uint16_t* b = bo.data() + (size_t)prow * (s->nb + 1);
      for (int t = 0; t < s->nb; ++t)
        for (int64_t e = (int64_t)rp[(size_t)r] + b[t]; e < (int64_t)rp[(size_t)r] + b[t + 1] && e < nnz; ++e)
          col[e] = pair_col(ent[e], t);
    }
  } else {
    std::vector<uint16_t> idx((size_t)nnz);
    if (nnz) HIP_TRY(c, hipMemcpy(idx.data(), isrc, idx.size() * 2, hipMemcpyDeviceToHost));
    for (int64_t i = 0; i < nnz; ++i) col[i] = idx[(size_t)i];
  }
  return RAD_OK;
}

extern "C" rad_status rad_store_export_bits(rad_ctx* c, const rad_store* s, uint32_t* words) {
  if (!c) return RAD_ERR_NULL;
  if (!s || !words) return fail(c, RAD_ERR_NULL, "null argument");
  if (!s->bits) return fail(c, RAD_ERR_PARAM, "store has no ReLU bits");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  HIP_TRY(c, hipMemcpy(words, s->bits, (size_t)s->steps * s->rows * s->bits_pitch * 4, hipMemcpyDeviceToHost));
  return RAD_OK;
}

extern "C" rad_status rad_store_import_bits(rad_ctx* c, rad_store* s, const uint32_t* words) {
  if (!c) return RAD_ERR_NULL;
  if (!s || !words) return fail(c, RAD_ERR_NULL, "null argument");
  if (!s->bits) return fail(c, RAD_ERR_PARAM, "store has no ReLU bits");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  HIP_TRY(c, hipMemcpy(s->bits, words, (size_t)s->steps * s->rows * s->bits_pitch * 4, hipMemcpyHostToDevice));
  return RAD_OK;
}

// draws the keep sets of every row and step of `s` into `bitmap`
// clear_max_seg = false when the caller has already zeroed the segment maxima of all its stores at once
static rad_status store_plan(rad_ctx* c, rad_store* s, const rad_sampling* sm, uint32_t* bitmap,
                             bool clear_max_seg = true, bool untimed = false) {
  if (s->scheme == RAD_EXACT || s->project()) return RAD_OK;
  PlanArgs a;
  a.seed_lo = (uint32_t)sm->seed; a.seed_hi = (uint32_t)(sm->seed >> 32);
  a.stream_id = sm->stream_id; a.step0 = sm->step;
  a.scheme = s->scheme;
  a.plan_rows = s->steps * s->plan_rows_per_step;
  a.rows_per_step = s->rows;
  a.cols = s->cols; a.k = s->k; a.k_pitch = s->k_pitch;
  a.thresh = (uint64_t)std::llround(s->p * 4294967296.0) >> c->key_shift;
  a.key_shift = c->key_shift;
  c->key_shift = 0;                 // the test hook serves one draw: it cannot be left on
  a.bitmap = bitmap; a.bm_pitch = s->bm_pitch;
  a.bucket_off = s->bucket_off; a.nb = s->nb;
  a.row_cnt = s->row_cnt; a.row_ptr = s->row_ptr;
  a.max_seg = s->max_seg;
  a.mult = s->mult;
  s->last_plan = *sm; s->planned = true;
  s->bitmap = bitmap;
  if (clear_max_seg) HIP_TRY(c, launch_fill_u32(reinterpret_cast<uint32_t*>(s->max_seg), 0u, 1, c->stream));
  if (untimed) {              // launches only: the timing wrapper may create events
    HIP_TRY(c, launch_plan(a, c->stream));
    if (s->counted_rows())
      HIP_TRY(c, launch_row_scan(s->row_cnt, s->row_ptr, s->steps * s->rows, s->capacity, s->overflow, c->stream));
    return RAD_OK;
  }
  HIP_TRY(c, timed(c, "plan", [&](const char**) { return launch_plan(a, c->stream); }));
  if (s->counted_rows()) {
    HIP_TRY(c, timed(c, "row_scan", [&](const char**) {
      return launch_row_scan(s->row_cnt, s->row_ptr, s->steps * s->rows, s->capacity, s->overflow, c->stream);
    }));
  }
  return RAD_OK;
}

static rad_status check_sampling(rad_ctx* c, const rad_sampling* sm, const rad_store* s) {
  if (!sm) return fail(c, RAD_ERR_NULL, "sampling is null");
  RAD_TRY(check_scheme(c, sm->scheme, sm->p));
  if (sm->scheme != s->scheme || sm->p != s->p) return fail(c, RAD_ERR_PARAM, "sampling does not match the store");
  return RAD_OK;
}

static rad_status store_pack(rad_ctx* c, rad_store* s, const void* x, int slot) {
  if (s->scheme == RAD_EXACT) {
    const size_t bytes = (size_t)s->rows * s->cols * s->elem();
    HIP_TRY(c, hipMemcpyAsync(static_cast<char*>(s->values) + (size_t)slot * bytes, x, bytes, hipMemcpyDeviceToDevice,
                              c->stream));
    return RAD_OK;
  }
  const StoreView v = store_view(s, slot);
  HIP_TRY(c, timed(c, s->dtype == kBF16 ? "pack_bf16" : "pack_f32",
                   [&](const char**) { return launch_pack(x, s->dtype, v, c->stream); }));
  return RAD_OK;
}

static rad_status project_forward(rad_ctx* c, rad_store* s, const rad_sampling* sm, const void* x, int slot = 0);

extern "C" rad_status rad_sample_pack(rad_ctx* c, const rad_sampling* sm, const void* x, rad_store* s,
                                      int32_t step_slot) {
  if (!c) return RAD_ERR_NULL;
  if (!s || !x) return fail(c, RAD_ERR_NULL, "null argument");
  RAD_TRY(check_sampling(c, sm, s));
  if (step_slot < 0 || step_slot >= s->steps) return fail(c, RAD_ERR_SHAPE, "step_slot out of range");
  if (s->steps != 1) return fail(c, RAD_ERR_UNSUPPORTED, "rad_sample_pack draws single-step stores only");
  if (s->project()) return project_forward(c, s, sm, x);
  void* bm = nullptr;
  if (s->scheme != RAD_EXACT) RAD_TRY(ws_get(c, WS_BITMAP, s->bitmap_words() * 4, &bm));
  RAD_TRY(store_plan(c, s, sm, static_cast<uint32_t*>(bm)));
  return store_pack(c, s, x, step_slot);
}

// rad_sample_pack for callers that must not allocate: the keep bitmap, which rad_sample_pack takes from a
// grow-only context workspace (hipMalloc on first use or growth), lies in the library's static device array.
// Same kernels, same results.  Nothing in the array has to start at zero: the plan kernel writes every word of
// every row that the pack kernel reads.
extern "C" rad_status rad_sample_pack_static(rad_ctx* c, const rad_sampling* sm, const void* x, rad_store* s) {
  if (!c) return RAD_ERR_NULL;
  if (!s || !x) return fail(c, RAD_ERR_NULL, "null argument");
  RAD_TRY(check_sampling(c, sm, s));
  if (s->steps != 1) return fail(c, RAD_ERR_UNSUPPORTED, "rad_sample_pack_static draws single-step stores only");
  if (s->project())
    return fail(c, RAD_ERR_UNSUPPORTED, "the projection schemes need workspaces that rad_sample_pack_static does not have");
  if (s->bitmap_words() > kScratchWords)
    return fail(c, RAD_ERR_CAPACITY, "rad_sample_pack_static: rows x ceil(cols/32) keep words exceed the static scratch (" +
                                     std::to_string(s->bitmap_words() * 4) + " > " +
                                     std::to_string((size_t)RAD_STATIC_SCRATCH_BYTES) + " bytes)");
  if (c->device < 0 || c->device >= kMaxDevices || !g_scratch[c->device])
    return fail(c, RAD_ERR_DEVICE, "static scratch was not resolved on this device");
  uint32_t* bm = g_scratch[c->device];
  if (s->scheme == RAD_EXACT) {
    HIP_TRY(c, hipMemcpyAsync(s->values, x, (size_t)s->rows * s->cols * s->elem(), hipMemcpyDeviceToDevice, c->stream));
    return RAD_OK;
  }
  RAD_TRY(store_plan(c, s, sm, bm, true, true));
  HIP_TRY(c, launch_pack(x, s->dtype, store_view(s, 0), c->stream));
  return RAD_OK;
}

// ------------------------------------------------------------ layer calls
static bool layer_matches(const rad_layer* L, const rad_store* s) {
  return L->batch == s->rows && L->d_in == s->cols && L->d_out == s->d_out && L->dtype == s->dtype &&
         (L->relu != 0) == (s->bits != nullptr);
}

static GemmArgs gemm_zero() { GemmArgs g; std::memset(&g, 0, sizeof(g)); return g; }

// alg_flops: what the operation needs by its definition when that is less than the 2 M N K the kernel
// executes (dW from a sampled store); 0 = the same
static rad_status run_gemm_call(rad_ctx* c, int dtype, int ak, int bk, int epi, const GemmArgs& g,
                                double alg_flops = 0.0) {
  const char* label = "gemm";
  if (c->timing) {              // the label decides whether this launch is bracketed by events
    GemmArgs probe = g; probe.dry_run = 1;
    if (launch_gemm(dtype, ak, bk, epi, probe, c->stream, &label) != hipSuccess) label = "gemm";
  }
  const size_t n_rec = c->recs.size();
  hipError_t e;
  if (c->timing && (c->filter.empty() || std::string(label).find(c->filter) != std::string::npos)) {
    // the launch carries its own start and end events: no event packets around it on the stream
    hipEvent_t ev[2];
    for (hipEvent_t& v : ev) {
      if (!c->pool.empty()) { v = c->pool.back(); c->pool.pop_back(); }
      else { hipError_t ce = hipEventCreate(&v); if (ce != hipSuccess) return hip_fail(c, ce, "event"); }
    }
    GemmArgs gt = g;
    gt.ev_start = ev[0]; gt.ev_stop = ev[1];
    const char* nm = label;
    e = launch_gemm(dtype, ak, bk, epi, gt, c->stream, &nm);
    if (e == hipSuccess) c->recs.push_back({nm, ev[0], ev[1], 0.0, 0.0});
  } else {
    e = launch_gemm(dtype, ak, bk, epi, g, c->stream, nullptr);
  }
  if (c->recs.size() > n_rec) {
    c->recs.back().exe_flops = 2.0 * g.M * g.N * g.K;
    c->recs.back().alg_flops = alg_flops > 0.0 ? alg_flops : c->recs.back().exe_flops;
  }
  if (e == hipErrorInvalidValue) return fail(c, RAD_ERR_UNSUPPORTED, "no GEMM kernel for this operand combination");
  if (e != hipSuccess) return hip_fail(c, e, "gemm launch");
  return RAD_OK;
}

// y = act(x W + bias [+ u V]); writes ReLU bits and, if `next`, the packed sample of y
static rad_status forward_gemm(rad_ctx* c, int dtype, int M, int N, int K, const void* x, int64_t ldx, const void* W,
                               const float* bias, int relu, void* y, uint32_t* bits, int bits_pitch,
                               const StoreView* next, const float* u, int64_t u_ld, int u_n, const float* V) {
  GemmArgs g = gemm_zero();
  g.M = M; g.N = N; g.K = K;
  g.A = x; g.lda = ldx; g.B = W; g.ldb = N;
  // A narrow output (the class scores) gives too few 256x256 tiles to fill the chip, and 256x64 tiles run at a
  // fifth of the MFMA rate: split K over several workgroups per tile; each stores fp32 partial sums to an array
  // of its own and one reduction kernel adds them, in a fixed order, with the bias.  Plain layers only.
  const int tiles = ((M + 255) / 256) * ((N + 255) / 256);
  if (dtype == kBF16 && !relu && !next && u_n == 0 && tiles < 128 && K >= 2048 && N % 4 == 0) {
    int splits = 256 / tiles;
    if (splits > 8) splits = 8;
    const int ks = ((K + splits - 1) / splits + 31) / 32 * 32;
    splits = (K + ks - 1) / ks;
    if (splits > 1) {
      // the rows of a partial array are padded to whole 256-column tiles: aligned stores whatever N is
      const int64_t pld = (int64_t)(N + 255) / 256 * 256;
      void* part = nullptr;
      RAD_TRY(ws_get(c, WS_SPLITK, (size_t)splits * M * pld * 4, &part));
      g.C = part; g.ldc = pld; g.c_dtype = kF32;
      g.k_split = ks; g.k_splits = splits; g.split_stride = (int64_t)M * pld;
      RAD_TRY(run_gemm_call(c, dtype, kOpK, kOpMN, kEpiStore, g));
      HIP_TRY(c, timed(c, "splitk_bias", [&](const char**) {
        return launch_splitk_bias(static_cast<const float*>(part), splits, M, N, bias, y, dtype, c->stream, pld);
      }));
      return RAD_OK;
    }
  }
  // fp32, few 64 x 64 tiles and a long contraction (a time step of the recurrent model: 128 x 1024 x 1024 is 32
  // tiles, each a chain of 64 K-slices): split K eight ways; one kernel then adds the partial sums and does the
  // epilogue's work (bias, input term, ReLU, bits), and the next store's sample is packed by the pack kernel
  const int tiles64 = ((M + 63) / 64) * ((N + 63) / 64);
  if (dtype == kF32 && tiles64 <= 64 && K >= 512) {
    // whole 32 x 32 tiles: one launch, K split over the waves of a workgroup and added in LDS
    GemmArgs gk = g;
    gk.bias = bias; gk.relu = relu; gk.y = y; gk.ldy = N; gk.bits = relu ? bits : nullptr; gk.bits_pitch = bits_pitch;
    gk.u = u; gk.u_ld = u_ld; gk.u_n = u_n; gk.V = V;
    if (gemm_f32_ks_ok(gk, false)) {
      HIP_TRY(c, timed(c, "gemm_f32_fwd_ks", [&](const char**) { return launch_gemm_f32_ks(gk, 1, c->stream); }));
      if (next)
        HIP_TRY(c, timed(c, "pack_f32", [&](const char**) { return launch_pack(y, kF32, *next, c->stream); }));
      return RAD_OK;
    }
    int splits = K / 128, want = 256 / tiles64;            // about one workgroup per CU
    if (want < 8) want = 8;
    if (want > 32) want = 32;
    if (splits > want) splits = want;
    const int ks = ((K + splits - 1) / splits + 31) / 32 * 32;   // whole K slices of the split kernels (32 deep)
    splits = (K + ks - 1) / ks;
    if (splits > 1) {
      void* part = nullptr;
      RAD_TRY(ws_get(c, WS_SPLITK, (size_t)splits * M * N * 4, &part));
      g.C = part; g.ldc = N; g.c_dtype = kF32;
      g.k_split = ks; g.k_splits = splits;
      RAD_TRY(run_gemm_call(c, dtype, kOpK, kOpMN, kEpiSplitK, g));
      HIP_TRY(c, timed(c, "splitk_fwd", [&](const char**) {
        return launch_splitk_fwd_f32(static_cast<const float*>(part), splits, M, N, bias, u, u_ld, u_n, V, relu,
                                     static_cast<float*>(y), relu ? bits : nullptr, bits_pitch, c->stream);
      }));
      if (next)
        HIP_TRY(c, timed(c, "pack_f32", [&](const char**) { return launch_pack(y, kF32, *next, c->stream); }));
      return RAD_OK;
    }
  }
  g.bias = bias; g.relu = relu; g.y = y; g.ldy = N; g.bits = relu ? bits : nullptr; g.bits_pitch = bits_pitch;
  if (next) { g.pack = 1; g.next = *next; }
  g.u = u; g.u_ld = u_ld; g.u_n = u_n; g.V = V;
  return run_gemm_call(c, dtype, kOpK, kOpMN, kEpiFwd, g);
}

// A k x N output gives few tiles when k is a small fraction of the layer width: split the K dimension (the
// batch) over several workgroups per tile; each stores its partial sums to an array of its own in a context
// workspace and launch_splitk_reduce_rows adds them in split order, so the result does not vary from run to run
// (bf16 ring kernels only).  The caller runs the GEMM on g and, when g->k_splits > 1, the reduction into the
// real output (*out, row_map, beta as recorded here).
struct SplitPlan { float* out = nullptr; int64_t ld = 0; const uint16_t* row_map = nullptr; int beta = 0; };
static rad_status split_k_for_few_tiles(rad_ctx* c, GemmArgs* g, SplitPlan* sp) {
  if (g->K < 512) return RAD_OK;
  const int tiles = ((g->M + 127) / 128) * ((g->N + 127) / 128);
  if (tiles >= 192) return RAD_OK;
  int splits = (512 + tiles - 1) / tiles;
  if (splits > 8) splits = 8;
  int ks = ((g->K + splits - 1) / splits + 31) / 32 * 32;
  if (ks < 256) ks = 256;
  splits = (g->K + ks - 1) / ks;
  if (splits <= 1) return RAD_OK;
  void* part = nullptr;
  RAD_TRY(ws_get(c, WS_SPLITK, (size_t)splits * g->M * g->N * 4, &part));
  sp->out = static_cast<float*>(g->C); sp->ld = g->ldc; sp->row_map = g->row_map; sp->beta = g->beta;
  g->k_split = ks; g->k_splits = splits; g->split_stride = (int64_t)g->M * g->N;
  g->C = part; g->ldc = g->N; g->row_map = nullptr; g->beta = 0;
  return RAD_OK;
}
static rad_status split_k_finish(rad_ctx* c, const GemmArgs& g, const SplitPlan& sp) {
  if (g.k_splits <= 1) return RAD_OK;
  HIP_TRY(c, timed(c, "splitk_reduce", [&](const char**) {
    return launch_splitk_reduce_rows(static_cast<const float*>(g.C), g.k_splits, g.split_stride, g.M, g.N, sp.row_map,
                                     sp.out, sp.ld, sp.beta, c->stream);
  }));
  return RAD_OK;
}

// ---- projection scheme (Section 3.2, P = R R^T / k; Appendix "Random projections for RAD")
// R [cols][k_pitch] and its transpose [k_pitch][cols] as +1 / -1 in the store's dtype, regenerated from the
// sampling parameters whenever they are needed (they are never kept: that is the memory saving)
static rad_status project_signs(rad_ctx* c, const rad_store* s, uint64_t seed, uint32_t stream_id, uint32_t step,
                                void** Rm, void** Rt) {
  const size_t bytes = (size_t)s->cols * s->k_pitch * s->elem();
  void* base = nullptr;
  RAD_TRY(ws_get(c, WS_PROJ_R, 2 * bytes, &base));
  HIP_TRY(c, timed(c, "fill", [&](const char**) {
    return launch_fill_u32(static_cast<uint32_t*>(base), 0u, (int64_t)(2 * bytes / 4), c->stream);
  }));
  *Rm = base; *Rt = static_cast<char*>(base) + bytes;
  HIP_TRY(c, timed(c, "sign_matrix", [&](const char**) {
    return launch_sign_matrix(*Rm, *Rt, s->dtype, s->cols, s->k, s->k_pitch, (uint32_t)seed, (uint32_t)(seed >> 32),
                              stream_id, step, c->stream);
  }));
  return RAD_OK;
}

// store (step slot `slot`) <- z = x R / sqrt(k): one more forward-family GEMM per layer.  The slots of a multi-step
// store are drawn with consecutive step numbers: slot q with the step of slot 0 plus q, which is what the backward
// pass regenerates R from.
static rad_status project_forward(rad_ctx* c, rad_store* s, const rad_sampling* sm, const void* x, int slot) {
  void* zdst = static_cast<char*>(s->values) + (size_t)slot * s->rows * s->k_pitch * s->elem();
  if (s->scheme == kProjectPerExample) {       // every example times its own matrix, signs drawn in the kernel
    HIP_TRY(c, timed(c, "project_rows_fwd", [&](const char**) {
      return launch_project_rows_fwd(x, s->dtype, s->rows, s->cols, s->k, s->k_pitch, s->scale, zdst,
                                     (uint32_t)sm->seed, (uint32_t)(sm->seed >> 32), sm->stream_id, sm->step, c->stream);
    }));
    s->proj_seed = sm->seed; s->proj_stream = sm->stream_id; s->proj_step = sm->step - (uint32_t)slot; s->proj_valid = true;
    return RAD_OK;
  }
  void *Rm = nullptr, *Rt = nullptr;
  RAD_TRY(project_signs(c, s, sm->seed, sm->stream_id, sm->step, &Rm, &Rt));
  GemmArgs g = gemm_zero();
  g.M = s->rows; g.N = s->k_pitch; g.K = s->cols;
  g.A = x; g.lda = s->cols; g.B = Rm; g.ldb = s->k_pitch;
  g.y = zdst; g.ldy = s->k_pitch; g.out_scale = s->scale;
  RAD_TRY(run_gemm_call(c, s->dtype, kOpK, kOpMN, kEpiFwd, g));
  s->proj_seed = sm->seed; s->proj_stream = sm->stream_id; s->proj_step = sm->step - (uint32_t)slot; s->proj_valid = true;
  return RAD_OK;
}

// dW = beta dW + R (z^T g) / sqrt(k): the k x N product first, then R times it
static rad_status project_dW(rad_ctx* c, const rad_store* s, const void* dy, int N, const uint32_t* bits,
                             int bits_pitch, float* dW, int beta, int slot = 0) {
  if (!s->proj_valid) return fail(c, RAD_ERR_PARAM, "the store holds no projection yet");
  const void* zsrc = static_cast<const char*>(s->values) + (size_t)slot * s->rows * s->k_pitch * s->elem();
  const uint32_t step = s->proj_step + (uint32_t)slot;
  if (s->scheme == kProjectPerExample) {
    // x~ = z R_b^T / sqrt(k) row by row into a transient dense operand (one layer's worth, reused), then the
    // dense contraction x~^T g
    void* dense = nullptr;
    RAD_TRY(ws_get(c, WS_DENSE, (size_t)s->rows * s->cols * s->elem(), &dense));
    HIP_TRY(c, timed(c, "project_rows_bwd", [&](const char**) {
      return launch_project_rows_bwd(zsrc, s->dtype, s->rows, s->cols, s->k, s->k_pitch, s->scale, dense,
                                     (uint32_t)s->proj_seed, (uint32_t)(s->proj_seed >> 32), s->proj_stream,
                                     step, c->stream);
    }));
    GemmArgs g = gemm_zero();
    g.M = s->cols; g.N = N; g.K = s->rows;
    g.A = dense; g.lda = s->cols;
    g.B = dy; g.ldb = N; g.b_mask = bits; g.b_mask_pitch = bits_pitch;
    g.C = dW; g.ldc = N; g.beta = beta; g.c_dtype = kF32;
    return run_gemm_call(c, s->dtype, kOpMN, kOpMN, kEpiStore, g);
  }
  void *Rm = nullptr, *Rt = nullptr;
  RAD_TRY(project_signs(c, s, s->proj_seed, s->proj_stream, step, &Rm, &Rt));
  void *T = nullptr, *Tb = nullptr;
  RAD_TRY(ws_get(c, WS_PROJ_T, (size_t)s->k_pitch * N * 4, &T));
  RAD_TRY(ws_get(c, WS_PROJ_TB, (size_t)s->k_pitch * N * s->elem(), &Tb));
  GemmArgs g = gemm_zero();
  g.M = s->k_pitch; g.N = N; g.K = s->rows;
  g.A = zsrc; g.lda = s->k_pitch;
  g.B = dy; g.ldb = N; g.b_mask = bits; g.b_mask_pitch = bits_pitch;
  g.C = T; g.ldc = N; g.beta = 0; g.c_dtype = kF32;
  SplitPlan sp;
  if (s->dtype == kBF16) RAD_TRY(split_k_for_few_tiles(c, &g, &sp));
  RAD_TRY(run_gemm_call(c, s->dtype, kOpMN, kOpMN, kEpiStore, g));
  RAD_TRY(split_k_finish(c, g, sp));
  HIP_TRY(c, timed(c, "scale_cast", [&](const char**) {
    return launch_scale_cast(static_cast<const float*>(T), Tb, s->dtype, (int64_t)s->k_pitch * N, s->scale, c->stream);
  }));
  GemmArgs h = gemm_zero();
  h.M = s->cols; h.N = N; h.K = s->k_pitch;
  h.A = Rt; h.lda = s->cols;
  h.B = Tb; h.ldb = N;
  h.C = dW; h.ldc = N; h.beta = beta; h.c_dtype = kF32;
  return run_gemm_call(c, s->dtype, kOpMN, kOpMN, kEpiStore, h);
}

// What the backward kernels read: the store itself, or, for an index-free store, its transient rebuild: the
// keep bitmap is drawn again from the recorded sampling parameters and the (value, column) entries (bf16) or
// the columns (fp32) are written to a context workspace that lives until the next rebuild.
static rad_status backward_view(rad_ctx* c, const rad_store* cs, int slot, StoreView* out) {
  *out = store_view(cs, slot);
  if (!cs->index_free) return RAD_OK;
  rad_store* s = const_cast<rad_store*>(cs);       // the plan tables are rewritten with the values they hold
  if (!s->planned) return fail(c, RAD_ERR_PARAM, "the index-free store has not been sampled yet");
  if (s->steps != 1) return fail(c, RAD_ERR_UNSUPPORTED, "index-free multi-step stores are read inside rad_train_step only");
  void* bm = nullptr;
  RAD_TRY(ws_get(c, WS_BITMAP, s->bitmap_words() * 4, &bm));
  const rad_sampling sm = s->last_plan;
  RAD_TRY(store_plan(c, s, &sm, static_cast<uint32_t*>(bm), false));
  *out = store_view(s, slot);
  void* ws = nullptr;
  const size_t bytes = s->dtype == kBF16 ? (size_t)(s->capacity + kPairPad) * 4 : (size_t)s->capacity * 2;
  RAD_TRY(ws_get(c, WS_REINDEX, bytes, &ws));
  const StoreView v = *out;
  HIP_TRY(c, timed(c, "reindex", [&](const char**) {
    return launch_reindex(v, s->dtype, static_cast<uint32_t*>(ws), static_cast<uint16_t*>(ws), c->stream);
  }));
  if (s->dtype == kBF16) { out->values = ws; out->paired = 1; }
  else out->indices = static_cast<uint16_t*>(ws);
  return RAD_OK;
}

extern "C" rad_status rad_store_set_index_free(rad_ctx* c, rad_store* s, int32_t on) {
  if (!c) return RAD_ERR_NULL;
  if (!s) return fail(c, RAD_ERR_NULL, "store is null");
  if (!s->per_entry()) return fail(c, RAD_ERR_UNSUPPORTED, "index-free storage serves stores with per-entry columns");
  if (s->steps != 1 && s->dtype != kF32)
    return fail(c, RAD_ERR_UNSUPPORTED, "index-free multi-step stores are fp32 only");
  if ((on != 0) == s->index_free) return RAD_OK;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (s->values) (void)hipFree(s->values);
  if (s->indices) (void)hipFree(s->indices);
  s->values = nullptr; s->indices = nullptr;
  s->index_free = on != 0; s->planned = false;
  const size_t vbytes = s->paired() ? (size_t)(s->capacity + kPairPad) * 4 : (size_t)s->capacity * s->elem();
  if (hipMalloc(&s->values, vbytes ? vbytes : 16) != hipSuccess) return fail(c, RAD_ERR_DEVICE, "store allocation failed");
  if (!s->paired() && !s->index_free &&
      hipMalloc(reinterpret_cast<void**>(&s->indices), (size_t)s->capacity * 2 + 16) != hipSuccess)
    return fail(c, RAD_ERR_DEVICE, "store allocation failed");
  return RAD_OK;
}

static int sparse_prefetch_for(const rad_store* s, int lanes_per_row) {
  const double pi = s->scheme == RAD_BERNOULLI ? s->p : (double)s->k / (double)s->cols;
  const double mean = pi * (s->cols < kBucket ? s->cols : kBucket);
  return (int)std::ceil((mean + 6.0 * std::sqrt(mean)) / lanes_per_row);   // overflow beyond this is rare and handled apart
}

// whether dW_gemm with rows of dy dy_ld apart runs the store-fed kernel with a split K (the one path that takes a
// pitched dy): a bf16 store with its own columns per row, sparse enough for that kernel, too few tiles to fill the chip
static bool dw_pitched_ok(const rad_store* s, int N, int dy_ld) {
  if (dy_ld <= N || dy_ld % 256 || s->dtype != kBF16 || s->project() || s->steps != 1) return false;
  if (s->scheme == RAD_EXACT || s->scheme == RAD_FIXEDK_SHARED) return false;
  if (sparse_prefetch_for(s, 8) > gemm_bf16_sparse_max_prefetch()) return false;
  const int64_t tiles = ((s->cols + 255) / 256) * (int64_t)(dy_ld / 256);
  return tiles < 128 && 256 / tiles >= 2 && s->rows >= 2048;
}

// dW = beta dW + store(slot)^T (dy masked by bits)
// n_slots > 1: the contraction runs over that many consecutive step slots of a multi-step store at once (their
// rows lie one after another in the store; dy then holds the rows of all those steps in the same order); only for
// stores whose rows are planned one by one and kept with their indices
// dy_ld > N (see dw_pitched_ok): the rows of dy are dy_ld apart, a multiple of 256, and zero past column N; the
// contraction then runs on whole tiles of dy_ld columns and only the reduction of its split-K partial sums knows N
static bool dw_pitched_ok(const rad_store* s, int N, int dy_ld);
static rad_status dW_gemm(rad_ctx* c, const rad_store* s, int slot, const void* dy, int N, const uint32_t* bits,
                          int bits_pitch, float* dW, int beta, int n_slots = 1, int dy_ld = 0) {
  if (dy_ld > 0 && dy_ld != N && (n_slots != 1 || bits || !dw_pitched_ok(s, N, dy_ld)))
    return fail(c, RAD_ERR_PARAM, "pitched dy outside the split-K path of dW");
  const int n_out = N;
  if (dy_ld > N) N = dy_ld;
  if (s->project()) return project_dW(c, s, dy, N, bits, bits_pitch, dW, beta, slot);
  GemmArgs g = gemm_zero();
  g.N = N; g.K = s->rows * n_slots;
  g.B = dy; g.ldb = N; g.b_mask = bits; g.b_mask_pitch = bits_pitch;
  g.C = dW; g.ldc = N; g.beta = beta; g.c_dtype = kF32;
  if (s->scheme == RAD_EXACT) {
    g.M = s->cols;
    g.A = static_cast<const char*>(s->values) + (size_t)slot * s->rows * s->cols * s->elem(); g.lda = s->cols;
    return run_gemm_call(c, s->dtype, kOpMN, kOpMN, kEpiStore, g);
  }
  if (s->scheme == RAD_FIXEDK_SHARED) {
    // compact problem: only the k sampled rows of dW are touched, the rest is zero
    if (!beta)
      HIP_TRY(c, timed(c, "fill", [&](const char**) {
        return launch_fill_u32(reinterpret_cast<uint32_t*>(dW), 0u, (int64_t)s->cols * N, c->stream);
      }));
    g.M = s->k; g.m_load = s->k_pitch;     // the operand is readable (zeros) up to the padded width
    g.A = static_cast<const char*>(s->values) + (size_t)slot * s->rows * s->k_pitch * s->elem(); g.lda = s->k_pitch;
    g.row_map = s->indices + (size_t)slot * s->k;
    g.beta = 1;
    SplitPlan sp;
    if (s->dtype == kBF16) RAD_TRY(split_k_for_few_tiles(c, &g, &sp));
    RAD_TRY(run_gemm_call(c, s->dtype, kOpMN, kOpMN, kEpiStore, g));
    return split_k_finish(c, g, sp);
  }
  g.M = s->cols;
  if (s->index_free && s->steps > 1) {
    // a multi-step store that keeps values only (the recurrent model): the keep bitmap of the step's own plan is
    // still there, and x~ of the chunk is rebuilt from it as a transient dense operand
    if (!s->bitmap || s->dtype != kF32) return fail(c, RAD_ERR_PARAM, "the index-free store has no current draw");
    StoreView v = store_view(s, slot);
    v.rows = s->rows * n_slots;
    void* dense = nullptr;
    RAD_TRY(ws_get(c, WS_DENSE, (size_t)v.rows * s->cols * 4, &dense));
    HIP_TRY(c, timed(c, "unpack", [&](const char**) { return launch_unpack_bitmap(v, kF32, dense, c->stream); }));
    g.K = v.rows; g.A = dense; g.lda = s->cols;
    const double kept = s->scheme == RAD_BERNOULLI ? s->p * (double)v.rows * s->cols : (double)v.rows * s->k;
    return run_gemm_call(c, kF32, kOpMN, kOpMN, kEpiStore, g, 2.0 * kept * N);
  }
  RAD_TRY(backward_view(c, s, slot, &g.sa));
  g.sa.rows = s->rows * n_slots;
  g.sparse_prefetch = sparse_prefetch_for(s, s->dtype == kBF16 ? 8 : 16);
  // 2 N flops per kept entry (expected number for Bernoulli draws)
  const double kept = s->scheme == RAD_BERNOULLI ? s->p * (double)s->rows * s->cols : (double)s->rows * s->k;
  const double alg = 2.0 * kept * N;
  if (s->dtype == kF32 && n_slots > 1) {
    // several steps at once (fp32, the recurrent model): the fp32 kernel's sparse loader pays per K-slice, so a
    // long contraction is cheaper from a transient dense x~ of the chunk
    void* dense = nullptr;
    RAD_TRY(ws_get(c, WS_DENSE, (size_t)g.sa.rows * s->cols * 4, &dense));
    HIP_TRY(c, timed(c, "unpack", [&](const char**) { return launch_unpack(g.sa, kF32, dense, c->stream); }));
    g.A = dense; g.lda = s->cols;
    return run_gemm_call(c, kF32, kOpMN, kOpMN, kEpiStore, g, alg);
  }
  // Wide bf16 layers whose shape the direct-to-LDS dense kernel takes (whole 256-row tiles of x~, an output width
  // of whole 16-byte vectors, no loader mask): the
  // store is unpacked into a transient dense x~ (one pass over 2 B D bytes) and contracted by that kernel, which
  // beats scattering every tile's entries into LDS in each of the N / 256 workgroups that need them (4096 x 4096,
  // fraction 0.1: 14 + 92 us against 121 us).
  const bool dense_pays = s->dtype == kBF16 && n_slots == 1 && !bits && s->cols % 256 == 0 && N % 8 == 0 &&
                          (s->cols / 256) * (int64_t)((N + 255) / 256) >= 128 && s->rows % 8 == 0 && s->rows >= 1024 &&
                          (size_t)s->cols * 2 <= 60 * 1024 && (reinterpret_cast<uintptr_t>(dy) & 15) == 0;
  if (s->dtype == kBF16 && (dense_pays || g.sparse_prefetch > gemm_bf16_sparse_max_prefetch())) {
    // (also: stores dense enough that scattering into LDS loses to a plain contraction whatever the shape.)
    // x~ is a transient dense operand, one layer's worth, reused by the next layer
    void* dense = nullptr;
    RAD_TRY(ws_get(c, WS_DENSE, (size_t)s->rows * s->cols * s->elem(), &dense));
    HIP_TRY(c, timed(c, "unpack", [&](const char**) { return launch_unpack(g.sa, s->dtype, dense, c->stream); }));
    g.A = dense; g.lda = s->cols;
    return run_gemm_call(c, s->dtype, kOpMN, kOpMN, kEpiStore, g, alg);
  }
  bool split = false;
  if (s->dtype == kBF16) {
    // A narrow dW (few output columns) gives too few 256x256 tiles to fill the chip, and 256x64 tiles run at
    // a fifth of the MFMA rate: split the batch over several workgroups per tile instead; each writes its
    // partial sums to an array of its own and a reduction kernel adds them in a fixed order.
    const int tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (tiles < 128 && g.K >= 2048) {
      int splits = 256 / tiles;
      if (splits > 8) splits = 8;
      const int ks = ((g.K + splits - 1) / splits + 31) / 32 * 32;
      splits = (g.K + ks - 1) / ks;
      if (splits > 1) {
        void* part = nullptr;
        RAD_TRY(ws_get(c, WS_SPLITK, (size_t)splits * g.M * g.N * 4, &part));
        g.k_split = ks; g.k_splits = splits; g.split_stride = (int64_t)g.M * g.N;
        g.C = part; g.beta = 0;
        split = true;
      }
    }
  }
  RAD_TRY(run_gemm_call(c, s->dtype, kOpSparse, kOpMN, kEpiStore, g, alg));
  if (split && n_out != N)
    HIP_TRY(c, timed(c, "splitk_reduce", [&](const char**) {
      return launch_splitk_reduce_rows(static_cast<const float*>(g.C), g.k_splits, g.split_stride, g.M, n_out, nullptr, dW,
                                       n_out, beta, c->stream, N);
    }));
  else if (split)
    HIP_TRY(c, timed(c, "splitk_reduce", [&](const char**) {
      return launch_splitk_reduce(static_cast<const float*>(g.C), g.k_splits, g.split_stride, dW, beta, c->stream);
    }));
  if (s->dtype == kBF16) {
    // the bf16 kernel keeps a fixed number of entries per (row, bucket) in registers; the rest, if any, here
    const int cap = gemm_bf16_sparse_cap(g.sparse_prefetch);
    HIP_TRY(c, timed(c, "dw_overflow", [&](const char**) {
      return launch_dw_overflow(g.sa, s->rows, dy, s->dtype, n_out, bits, bits_pitch, dW, cap, s->max_seg, c->stream, N);
    }));
  }
  return RAD_OK;
}

// dX = (dy masked by bits) W^T
// (dy masked by bits) W^T, optionally masked on the way out by the ReLU bits of the layer below, so that
// the chain hands g = dL/dh to the next dW and dX without loader masks
static rad_status dX_gemm(rad_ctx* c, int dtype, int M, int d_in, int d_out, const void* dy, const uint32_t* bits,
                          int bits_pitch, const void* W, void* dX, const uint32_t* out_bits = nullptr,
                          int out_pitch = 0, int dy_ld = 0) {
  GemmArgs g = gemm_zero();
  g.M = M; g.N = d_in; g.K = d_out;
  g.A = dy; g.lda = dy_ld > 0 ? dy_ld : d_out; g.a_mask = bits; g.a_mask_pitch = bits_pitch;
  g.B = W; g.ldb = d_out;
  // fp32 with few tiles and a long contraction: split K, then add the partial sums under the output mask
  const int tiles64 = ((M + 63) / 64) * ((d_in + 63) / 64);
  if (dtype == kF32 && tiles64 <= 64 && d_out >= 512) {
    GemmArgs gk = g;
    gk.y = dX; gk.ldy = d_in; gk.c_mask = out_bits; gk.c_mask_pitch = out_pitch;
    if (gemm_f32_ks_ok(gk, true)) {
      HIP_TRY(c, timed(c, "gemm_f32_dx_ks", [&](const char**) { return launch_gemm_f32_ks(gk, 2, c->stream); }));
      return RAD_OK;
    }
    int splits = d_out / 128;
    if (splits > 8) splits = 8;
    const int ks = ((d_out + splits - 1) / splits + 31) / 32 * 32;   // whole K slices of the split kernels (32 deep)
    splits = (d_out + ks - 1) / ks;
    if (splits > 1) {
      void* part = nullptr;
      RAD_TRY(ws_get(c, WS_SPLITK, (size_t)splits * M * d_in * 4, &part));
      g.C = part; g.ldc = d_in; g.c_dtype = kF32;
      g.k_split = ks; g.k_splits = splits;
      RAD_TRY(run_gemm_call(c, dtype, kOpK, kOpK, kEpiSplitK, g));
      HIP_TRY(c, timed(c, "splitk_reduce", [&](const char**) {
        return launch_splitk_reduce_masked(static_cast<const float*>(part), splits, M, d_in, out_bits, out_pitch,
                                           static_cast<float*>(dX), c->stream);
      }));
      return RAD_OK;
    }
  }
  g.C = dX; g.ldc = d_in; g.beta = 0; g.c_dtype = dtype;
  g.c_mask = out_bits; g.c_mask_pitch = out_pitch;
  return run_gemm_call(c, dtype, kOpK, kOpK, kEpiStore, g);
}

static rad_status colsum_call(rad_ctx* c, const void* dy, int dtype, int rows, int N, const uint32_t* bits,
                              int bits_pitch, const float* u, int64_t u_ld, int u_n, float* out_bias, float* out_u,
                              int beta, int u_block_rows = 0, int64_t u_block_stride = 0, int64_t dy_ld = 0) {
  int splits = rows / 64;
  if (rows <= 512) splits = 1;          // few rows: one launch that writes the sums itself
  if (splits < 1) splits = 1;
  if (splits > 32) splits = 32;
  void* part = nullptr;
  RAD_TRY(ws_get(c, WS_COLSUM, (size_t)splits * (u_n + 1) * N * 4, &part));
  HIP_TRY(c, timed(c, "colsum", [&](const char**) {
    return launch_colsum(dy, dtype, rows, N, bits, bits_pitch, u, u_ld, u_n, out_bias, out_u, beta,
                         static_cast<float*>(part), splits, c->stream, u_block_rows, u_block_stride, dy_ld);
  }));
  return RAD_OK;
}

// convolution pieces (defined with the CNN model below)
static rad_status conv_limits(rad_ctx* c, const rad_layer* L);
static rad_status conv_gemm(rad_ctx* c, int B, int ci, int co, int h, int w, int ks, const float* src, const float* W,
                            const float* bias, int relu, float* y, uint32_t* bits, int bits_pitch);
static rad_status conv_dW_call(rad_ctx* c, const rad_store* s, int B, int ci, int co, int h, int w, int ks, const float* g,
                               float* dW, float* dbias);
static rad_status conv_dX_call(rad_ctx* c, int B, int ci, int co, int h, int w, int ks, const float* g, const float* W,
                               float* dX);
// g = dy masked by the store's ReLU bits (dy itself for a layer without ReLU), in a context workspace
static rad_status conv_masked_dy(rad_ctx* c, const rad_layer* L, const rad_store* s, const void* dy, const float** g);

extern "C" rad_status rad_forward_sample(rad_ctx* c, const rad_layer* L, const rad_sampling* sm, const void* x,
                                         const void* W, const void* bias, void* y, rad_store* s) {
  if (!c) return RAD_ERR_NULL;
  RAD_TRY(check_layer(c, L));
  if (!x || !W || !y || !s) return fail(c, RAD_ERR_NULL, "null argument");
  if ((L->has_bias != 0) != (bias != nullptr)) return fail(c, RAD_ERR_NULL, "bias pointer does not match has_bias");
  if (!layer_matches(L, s)) return fail(c, RAD_ERR_SHAPE, "store was created for a different layer");
  if (L->kind == RAD_CONV2D) {
    // Section 4.2 (convolutional layers): the flattened input is sampled, the convolution itself is exact
    RAD_TRY(conv_limits(c, L));
    RAD_TRY(rad_sample_pack(c, sm, x, s, 0));
    return conv_gemm(c, (int)L->batch, L->c_in, L->c_out, L->h, L->w, L->kh, static_cast<const float*>(x),
                     static_cast<const float*>(W), static_cast<const float*>(bias), L->relu, static_cast<float*>(y),
                     s->bits, s->bits_pitch);
  }
  RAD_TRY(rad_sample_pack(c, sm, x, s, 0));
  return forward_gemm(c, L->dtype, (int)L->batch, (int)L->d_out, (int)L->d_in, x, L->d_in, W,
                      static_cast<const float*>(bias), L->relu, y, s->bits, s->bits_pitch, nullptr, nullptr, 0, 0,
                      nullptr);
}

extern "C" rad_status rad_backward_dW(rad_ctx* c, const rad_layer* L, const rad_store* s, const void* dy, float* dW,
                                      float* dbias, float beta) {
  if (!c) return RAD_ERR_NULL;
  RAD_TRY(check_layer(c, L));
  if (!s || !dy || !dW) return fail(c, RAD_ERR_NULL, "null argument");
  if (!layer_matches(L, s)) return fail(c, RAD_ERR_SHAPE, "store was created for a different layer");
  if (beta != 0.f && beta != 1.f) return fail(c, RAD_ERR_PARAM, "beta must be 0 or 1");
  if (s->steps != 1) return fail(c, RAD_ERR_UNSUPPORTED, "multi-step stores belong to rad_train_step");
  if (L->kind == RAD_CONV2D) {
    RAD_TRY(conv_limits(c, L));
    if (beta != 0.f) return fail(c, RAD_ERR_UNSUPPORTED, "conv gradients are written, not accumulated (beta = 0)");
    if (s->project()) return fail(c, RAD_ERR_UNSUPPORTED, "the projection schemes serve linear layers only");
    const float* g = nullptr;
    RAD_TRY(conv_masked_dy(c, L, s, dy, &g));
    return conv_dW_call(c, s, (int)L->batch, L->c_in, L->c_out, L->h, L->w, L->kh, g, dW, dbias);
  }
  RAD_TRY(dW_gemm(c, s, 0, dy, (int)L->d_out, s->bits, s->bits_pitch, dW, beta != 0.f));
  if (dbias)
    RAD_TRY(colsum_call(c, dy, L->dtype, (int)L->batch, (int)L->d_out, s->bits, s->bits_pitch, nullptr, 0, 0, dbias,
                        nullptr, beta != 0.f));
  return RAD_OK;
}

extern "C" rad_status rad_backward_dX(rad_ctx* c, const rad_layer* L, const rad_store* s, const void* dy,
                                      const void* W, void* dX) {
  if (!c) return RAD_ERR_NULL;
  RAD_TRY(check_layer(c, L));
  if (!s || !dy || !W || !dX) return fail(c, RAD_ERR_NULL, "null argument");
  if (!layer_matches(L, s)) return fail(c, RAD_ERR_SHAPE, "store was created for a different layer");
  if (L->kind == RAD_CONV2D) {
    RAD_TRY(conv_limits(c, L));
    const float* g = nullptr;
    RAD_TRY(conv_masked_dy(c, L, s, dy, &g));
    return conv_dX_call(c, (int)L->batch, L->c_in, L->c_out, L->h, L->w, L->kh, g, static_cast<const float*>(W),
                        static_cast<float*>(dX));
  }
  return dX_gemm(c, L->dtype, (int)L->batch, (int)L->d_in, (int)L->d_out, dy, s->bits, s->bits_pitch, W, dX);
}

static rad_status softmax_call(rad_ctx* c, const void* logits, const int32_t* labels, int rows, int classes, int dtype,
                               void* dlogits, float* loss_dev, int dz_ld = 0) {
  void* rl = nullptr;
  RAD_TRY(ws_get(c, WS_ROWLOSS, (size_t)rows * 4, &rl));
  HIP_TRY(c, timed(c, "softmax_ce", [&](const char**) {
    return launch_softmax_ce(logits, labels, rows, classes, dtype, dlogits, static_cast<float*>(rl), loss_dev,
                             c->stream, dz_ld);
  }));
  return RAD_OK;
}

extern "C" rad_status rad_softmax_ce(rad_ctx* c, const void* logits, const int32_t* labels, int64_t rows,
                                     int64_t classes, int32_t dtype, void* dlogits, float* loss_dev) {
  if (!c) return RAD_ERR_NULL;
  if (!logits || !labels || !dlogits || !loss_dev) return fail(c, RAD_ERR_NULL, "null argument");
  if (rows < 1 || classes < 1 || rows > (1 << 24) || classes > (1 << 24)) return fail(c, RAD_ERR_SHAPE, "bad shape");
  if (dtype != RAD_F32 && dtype != RAD_BF16) return fail(c, RAD_ERR_PARAM, "unknown dtype");
  return softmax_call(c, logits, labels, (int)rows, (int)classes, dtype, dlogits, loss_dev);
}

// ------------------------------------------------------------------ parameter updates
extern "C" rad_status rad_optimizer_step(rad_ctx* c, const rad_optimizer* opt, int64_t t, int32_t dtype,
                                         int32_t n_tensors, const int64_t* counts, void* const* params,
                                         const void* const* grads, void* const* m, void* const* v,
                                         void* const* master) {
  if (!c) return RAD_ERR_NULL;
  if (!opt || !counts || !params || !grads) return fail(c, RAD_ERR_NULL, "null argument");
  if (opt->kind != RAD_SGD && opt->kind != RAD_ADAM) return fail(c, RAD_ERR_PARAM, "unknown optimiser kind");
  if (dtype != RAD_F32 && dtype != RAD_BF16) return fail(c, RAD_ERR_PARAM, "unknown dtype");
  const bool adam = opt->kind == RAD_ADAM;
  if (n_tensors < 0) return fail(c, RAD_ERR_SHAPE, "negative tensor count");
  if (t < 1) return fail(c, RAD_ERR_PARAM, "step numbers start at 1");
  if (!(opt->lr > 0.0) || !std::isfinite(opt->lr) || !(opt->l2 >= 0.0) || !std::isfinite(opt->l2))
    return fail(c, RAD_ERR_PARAM, "lr must be positive and l2 non-negative");
  if (adam && (!(opt->beta1 >= 0.0 && opt->beta1 < 1.0) || !(opt->beta2 >= 0.0 && opt->beta2 < 1.0) ||
               !(opt->eps > 0.0) || !std::isfinite(opt->eps)))
    return fail(c, RAD_ERR_PARAM, "Adam needs 0 <= beta < 1 and eps > 0");
  if (adam && (!m || !v)) return fail(c, RAD_ERR_NULL, "Adam needs the moment arrays");
  if (dtype == RAD_BF16 && !master) return fail(c, RAD_ERR_NULL, "bf16 parameters need fp32 master copies");
  for (int i = 0; i < n_tensors; ++i) {
    if (counts[i] < 0) return fail(c, RAD_ERR_SHAPE, "negative element count");
    if (counts[i] == 0) continue;
    if (!params[i] || !grads[i] || (adam && (!m[i] || !v[i])) || (dtype == RAD_BF16 && !master[i]))
      return fail(c, RAD_ERR_NULL, "null tensor pointer");
  }
  OptimArgs a;
  a.lr = (float)opt->lr; a.l2 = (float)opt->l2;
  a.beta1 = adam ? (float)opt->beta1 : 0.f; a.beta2 = adam ? (float)opt->beta2 : 0.f; a.eps = adam ? (float)opt->eps : 0.f;
  a.omb1 = adam ? (float)(1.0 - opt->beta1) : 0.f; a.omb2 = adam ? (float)(1.0 - opt->beta2) : 0.f;
  a.inv_bc1 = adam ? (float)(1.0 / (1.0 - std::pow(opt->beta1, (double)t))) : 1.f;
  a.inv_bc2 = adam ? (float)(1.0 / (1.0 - std::pow(opt->beta2, (double)t))) : 1.f;
  for (int i = 0; i < n_tensors; ++i) {
    if (counts[i] == 0) continue;
    float* w = static_cast<float*>(dtype == RAD_BF16 ? master[i] : params[i]);
    uint16_t* lo = dtype == RAD_BF16 ? static_cast<uint16_t*>(params[i]) : nullptr;
    HIP_TRY(c, timed(c, adam ? "optim_adam" : "optim_sgd", [&](const char**) {
      return launch_optim(adam, w, lo, static_cast<const float*>(grads[i]), adam ? static_cast<float*>(m[i]) : nullptr,
                          adam ? static_cast<float*>(v[i]) : nullptr, counts[i], a, c->stream);
    }));
  }
  return RAD_OK;
}

// ------------------------------------------------------------------ reaction-diffusion study
struct PdeLayout { int64_t cap; size_t vals_bytes, rows_bytes, flags_bytes, total; };

static rad_status pde_layout(rad_ctx* c, const rad_pde_grid* g, double p, int32_t problems, PdeLayout* out) {
  if (!g) return fail(c, RAD_ERR_NULL, "grid is null");
  if (g->n < 2 || g->n > 32 || g->steps < 1 || problems < 1) return fail(c, RAD_ERR_SHAPE, "2 <= n <= 32, steps >= 1, problems >= 1");
  const double cells = (double)(g->n - 1) * (g->n - 1);
  if (cells * ((double)g->steps + 1.0) >= 4294967296.0) return fail(c, RAD_ERR_SHAPE, "steps (n-1)^2 must stay below 2^32");
  if (!(p > 0.0) || p > 1.0) return fail(c, RAD_ERR_PARAM, "p must be in (0, 1]");
  if (!(g->D > 0.0) || !(g->dt > 0.0) || g->D * g->dt * (double)g->n * (double)g->n > 0.25)
    return fail(c, RAD_ERR_PARAM, "D dt n^2 must be positive and at most 1/4");
  // each of the 16 waves of a problem (two grid rows, at most 62 interior entries) appends to a run of its own
  const double total = 62.0 * ((double)g->steps + 1.0);
  double cap = std::ceil(total * p + 8.0 * std::sqrt(total * p * (1.0 - p))) + 64.0;
  if (cap > total) cap = total;
  out->cap = (int64_t)cap;
  auto up = [](size_t b) { return (b + 255) / 256 * 256; };
  out->vals_bytes = up((size_t)problems * 16 * (size_t)out->cap * 8);
  out->rows_bytes = up((size_t)problems * 16 * 4);
  out->flags_bytes = up((size_t)problems * 4);
  out->total = out->vals_bytes + out->rows_bytes + out->flags_bytes;
  return RAD_OK;
}

extern "C" rad_status rad_pde_workspace_bytes(rad_ctx* c, const rad_pde_grid* g, double p, int32_t problems,
                                              uint64_t* bytes) {
  if (!c) return RAD_ERR_NULL;
  if (!bytes) return fail(c, RAD_ERR_NULL, "bytes is null");
  PdeLayout lay;
  RAD_TRY(pde_layout(c, g, p, problems, &lay));
  *bytes = lay.total;
  return RAD_OK;
}

extern "C" rad_status rad_pde_gradient(rad_ctx* c, const rad_pde_grid* g, int32_t problems, const double* theta,
                                       double p, uint64_t seed, uint32_t stream_id, void* workspace,
                                       uint64_t workspace_bytes, double* loss, double* grad, int64_t* stored) {
  if (!c) return RAD_ERR_NULL;
  if (!theta || !workspace || !loss || !grad) return fail(c, RAD_ERR_NULL, "null argument");
  PdeLayout lay;
  RAD_TRY(pde_layout(c, g, p, problems, &lay));
  if (workspace_bytes < lay.total) return fail(c, RAD_ERR_CAPACITY, "workspace smaller than rad_pde_workspace_bytes");
  if (reinterpret_cast<uintptr_t>(workspace) & 7) return fail(c, RAD_ERR_PARAM, "workspace must be 8-byte aligned");
  char* base = static_cast<char*>(workspace);
  double* vals = reinterpret_cast<double*>(base);
  uint32_t* rows = reinterpret_cast<uint32_t*>(base + lay.vals_bytes);
  int* flags = reinterpret_cast<int*>(base + lay.vals_bytes + lay.rows_bytes);
  HIP_TRY(c, timed(c, "pde", [&](const char**) {
    return launch_pde(problems, g->n, g->steps, g->D, g->dt, p, (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, theta,
                      vals, lay.cap, rows, flags, loss, grad, stored, c->stream);
  }));
  std::vector<int> host((size_t)problems);
  HIP_TRY(c, hipMemcpyAsync(host.data(), flags, (size_t)problems * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int f : host)
    if (f) return fail(c, RAD_ERR_CAPACITY, "a draw kept more entries than the workspace holds");
  return RAD_OK;
}

// ------------------------------------------------------------------ path sampling on a graph
extern "C" rad_status rad_path_sample_gradient(rad_ctx* c, const rad_graph* g, int32_t y, const int32_t* inputs,
                                               int32_t n_inputs, int32_t k, uint64_t seed, uint32_t stream_id,
                                               double* adjoint, uint32_t* reached) {
  if (!c) return RAD_ERR_NULL;
  if (!g || !inputs || !adjoint || !reached) return fail(c, RAD_ERR_NULL, "null argument");
  if (!g->level_ptr || !g->succ_ptr || (g->n_edges > 0 && (!g->succ || !g->partial))) return fail(c, RAD_ERR_NULL, "null graph array");
  if (g->n_vertices < 1 || g->n_vertices > (1 << 30) || g->n_levels < 1 || g->n_edges < 0 || g->n_edges > 0x7fffffffLL)
    return fail(c, RAD_ERR_SHAPE, "bad graph size");
  if (y < 0 || y >= g->n_vertices || n_inputs < 1 || n_inputs > g->n_vertices) return fail(c, RAD_ERR_SHAPE, "bad y or inputs");
  if (k < 1 || k > 65536) return fail(c, RAD_ERR_PARAM, "k must be in 1 .. 65536");
  if (g->level_ptr[0] != 0 || g->level_ptr[g->n_levels] != g->n_vertices) return fail(c, RAD_ERR_SHAPE, "levels must cover the vertices");
  for (int l = 0; l < g->n_levels; ++l)
    if (g->level_ptr[l + 1] < g->level_ptr[l]) return fail(c, RAD_ERR_SHAPE, "level_ptr must not decrease");
  void* flag = nullptr;
  RAD_TRY(ws_get(c, WS_ROWLOSS, 4, &flag));
  HIP_TRY(c, timed(c, "path_sampling", [&](const char**) {
    return launch_path_sampling(g->n_vertices, g->n_levels, g->level_ptr, g->n_edges, g->succ_ptr, g->succ, g->partial, y,
                                inputs, n_inputs, k, (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, adjoint, reached,
                                static_cast<int*>(flag), c->stream);
  }));
  int bad = 0;
  HIP_TRY(c, hipMemcpyAsync(&bad, flag, 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (bad) return fail(c, RAD_ERR_PARAM, "graph arrays are inconsistent");
  return RAD_OK;
}

// ------------------------------------------------------------------ models
enum ModelKind { kMlp = 0, kRnn = 1, kCnn = 2 };
constexpr int kRnnChunk = 8;            // time steps whose recurrent dW is one contraction over steps x batch

struct rad_model {
  int kind = kMlp;
  int dtype = 0, scheme = 0, has_bias = 0;
  double p = 1.0;
  int64_t batch = 0;
  std::vector<int64_t> dims;            // MLP widths
  std::vector<rad_store*> stores;
  void* act[2] = {nullptr, nullptr};    // transient dense activations (ping-pong)
  void* dyb[2] = {nullptr, nullptr};    // transient upstream gradients (ping-pong)
  void* logits = nullptr;
  int last_pitch = 0;                   // MLP: row pitch of the loss gradient when it is padded to whole tiles, else 0
  int* flags = nullptr;                 // [n stores] overflow flags, then [n stores] segment maxima
  // RNN
  int64_t T = 0, d_input = 0, hidden = 0, classes = 0;
  uint32_t* rnn_bits = nullptr;         // [T][batch][hidden/32]
  float* rnn_g = nullptr;               // [2][kRnnChunk][batch][hidden]: g of the time steps whose dW is formed together,
                                        // two chunks: one being read by the side stream, one being filled
  uint32_t* bitmap_ws = nullptr;        // keep bitmaps of every step (transient within a step)
  // CNN
  struct Conv { int ci, co, h, w, pool; uint32_t* arg; };
  std::vector<Conv> convs;
  int ksize = 0, fc_in = 0;
  void* buf[3] = {nullptr, nullptr, nullptr};   // transient dense activations / gradients
  size_t elem() const { return dtype == kBF16 ? 2 : 4; }
};

static rad_status model_share_flags(rad_ctx* c, rad_model* m);

extern "C" rad_status rad_model_destroy(rad_model* m) {
  if (!m) return RAD_ERR_NULL;
  for (rad_store* s : m->stores) if (s) rad_store_destroy(s);
  for (void* p : {m->act[0], m->act[1], m->dyb[0], m->dyb[1], m->logits, (void*)m->flags, (void*)m->rnn_bits, (void*)m->rnn_g, (void*)m->bitmap_ws,
                  m->buf[0], m->buf[1], m->buf[2]})
    if (p) (void)hipFree(p);
  for (auto& cv : m->convs) if (cv.arg) (void)hipFree(cv.arg);
  delete m;
  return RAD_OK;
}

extern "C" rad_status rad_model_set_index_free(rad_ctx* c, rad_model* m, int32_t on) {
  if (!c) return RAD_ERR_NULL;
  if (!m) return fail(c, RAD_ERR_NULL, "model is null");
  for (rad_store* s : m->stores)
    if (s->per_entry()) RAD_TRY(rad_store_set_index_free(c, s, on));
  return RAD_OK;
}

extern "C" int32_t rad_model_num_stores(const rad_model* m) { return m ? (int32_t)m->stores.size() : 0; }
extern "C" rad_store* rad_model_store(rad_model* m, int32_t l) {
  return (m && l >= 0 && l < (int32_t)m->stores.size()) ? m->stores[(size_t)l] : nullptr;
}
extern "C" const void* rad_model_logits(const rad_model* m) { return m ? m->logits : nullptr; }

extern "C" rad_status rad_model_export_pool_arg(rad_ctx* c, const rad_model* m, int32_t l, uint8_t* out) {
  if (!c) return RAD_ERR_NULL;
  if (!m || !out) return fail(c, RAD_ERR_NULL, "null argument");
  if (l < 0 || l >= (int32_t)m->convs.size() || !m->convs[(size_t)l].arg) return fail(c, RAD_ERR_PARAM, "layer has no max pool");
  const rad_model::Conv& cv = m->convs[(size_t)l];
  const size_t n = (size_t)m->batch * cv.co * (cv.h / 2) * (cv.w / 2);
  std::vector<uint32_t> words((n + 15) / 16);
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  HIP_TRY(c, hipMemcpy(words.data(), cv.arg, words.size() * 4, hipMemcpyDeviceToHost));
  for (size_t q = 0; q < n; ++q) out[q] = (uint8_t)((words[q / 16] >> (2 * (q % 16))) & 3u);
  return RAD_OK;
}

extern "C" rad_status rad_model_create_mlp(rad_ctx* c, int32_t dtype, int64_t batch, int32_t n_layers,
                                           const int64_t* dims, int32_t has_bias, int32_t scheme, double p,
                                           rad_model** out) {
  if (!c) return RAD_ERR_NULL;
  if (!out || !dims) return fail(c, RAD_ERR_NULL, "null argument");
  *out = nullptr;
  if (n_layers < 1 || n_layers > 64) return fail(c, RAD_ERR_SHAPE, "n_layers must be in [1, 64]");
  RAD_TRY(check_scheme(c, scheme, p));
  rad_model* m = new rad_model();
  m->kind = kMlp; m->dtype = dtype; m->scheme = scheme; m->p = p; m->batch = batch; m->has_bias = has_bias;
  m->dims.assign(dims, dims + n_layers + 1);
  int64_t widest = 0;
  for (int l = 0; l < n_layers; ++l) {
    rad_layer L; std::memset(&L, 0, sizeof(L));
    L.kind = RAD_LINEAR; L.dtype = dtype; L.batch = batch; L.d_in = dims[l]; L.d_out = dims[l + 1];
    L.relu = l < n_layers - 1; L.has_bias = has_bias;
    rad_store* s = nullptr;
    rad_status st = rad_store_create(c, &L, scheme, p, 1, &s);
    if (st != RAD_OK) { rad_model_destroy(m); return st; }
    m->stores.push_back(s);
    if (dims[l + 1] > widest) widest = dims[l + 1];
  }
  // A last layer whose width is not a multiple of 256 (class scores): its loss gradient is kept with rows padded to
  // whole tiles (zeros), so that dW of that layer runs on whole 256-column tiles of aligned rows; dX reads the same
  // rows and only the reduction of dW's split-K partial sums knows the real width.
  {
    const int64_t n_last = dims[n_layers], np = (n_last + 255) / 256 * 256;
    if (n_last % 256 != 0 && n_last % 8 == 0 && np / 8 <= 128 &&
        dw_pitched_ok(m->stores.back(), (int)n_last, (int)np)) {
      m->last_pitch = (int)np;
      if (np > widest) widest = np;
    }
  }
  const size_t bytes = (size_t)batch * widest * m->elem();
  bool ok = true;
  for (void** p2 : {&m->act[0], &m->act[1], &m->dyb[0], &m->dyb[1]}) ok = ok && hipMalloc(p2, bytes) == hipSuccess;
  ok = ok && hipMalloc(&m->logits, (size_t)batch * dims[n_layers] * m->elem()) == hipSuccess;
  if (!ok) { rad_model_destroy(m); return fail(c, RAD_ERR_DEVICE, "model allocation failed"); }
  { rad_status fs = model_share_flags(c, m); if (fs != RAD_OK) { rad_model_destroy(m); return fs; } }
  *out = m;
  return RAD_OK;
}

// The stores of a model keep their flags in one array of the model, so that a step clears the segment
// maxima of all of them with one launch and reads all overflow flags with one copy.
static rad_status model_share_flags(rad_ctx* c, rad_model* m) {
  const size_t n = m->stores.size();
  if (hipMalloc(reinterpret_cast<void**>(&m->flags), 2 * n * sizeof(int)) != hipSuccess)
    return fail(c, RAD_ERR_DEVICE, "model allocation failed");
  HIP_TRY(c, hipMemsetAsync(m->flags, 0, 2 * n * sizeof(int), c->stream));
  for (size_t l = 0; l < n; ++l) {
    rad_store* s = m->stores[l];
    if (s->overflow && !s->flags_external) (void)hipFree(s->overflow);
    s->overflow = m->flags + l; s->max_seg = m->flags + n + l; s->flags_external = true;
  }
  return RAD_OK;
}

static rad_status model_clear_max_seg(rad_ctx* c, rad_model* m) {
  const size_t n = m->stores.size();
  HIP_TRY(c, timed(c, "fill", [&](const char**) {
    return launch_fill_u32(reinterpret_cast<uint32_t*>(m->flags + n), 0u, (int64_t)n, c->stream);
  }));
  return RAD_OK;
}

// end of a step: with loss_host the step is waited for, the loss read back and a capacity overflow (also
// one left by earlier steps that were only enqueued) reported once; without it nothing waits
static rad_status step_finish(rad_ctx* c, rad_model* m, float* loss_host) {
  if (!loss_host) return RAD_OK;
  HIP_TRY(c, hipMemcpyAsync(loss_host, c->loss_dev, sizeof(float), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (m->scheme != RAD_BERNOULLI) return RAD_OK;
  std::vector<int> ov(m->stores.size(), 0);
  HIP_TRY(c, hipMemcpy(ov.data(), m->flags, ov.size() * sizeof(int), hipMemcpyDeviceToHost));
  for (int v : ov)
    if (v) {
      HIP_TRY(c, hipMemset(m->flags, 0, ov.size() * sizeof(int)));
      return fail(c, RAD_ERR_CAPACITY, "a Bernoulli draw exceeded a store's capacity");
    }
  return RAD_OK;
}

static rad_status mlp_step(rad_ctx* c, rad_model* m, const rad_sampling* sm, const void* x, const int32_t* labels,
                           void* const* params, void* const* grads, float* loss_host) {
  const int Lc = (int)m->stores.size();
  const int B = (int)m->batch;
  const int per = m->has_bias ? 2 : 1;
  for (int i = 0; i < Lc * per; ++i)
    if (!params[i] || !grads[i]) return fail(c, RAD_ERR_NULL, "null parameter or gradient pointer");
  auto Wp = [&](int l) { return params[l * per]; };
  auto bp = [&](int l) { return m->has_bias ? static_cast<const float*>(params[l * per + 1]) : nullptr; };
  size_t bm_words = 0;
  for (rad_store* s : m->stores) if (s->bitmap_words() > bm_words) bm_words = s->bitmap_words();
  void* bm = nullptr;
  if (bm_words) RAD_TRY(ws_get(c, WS_BITMAP, bm_words * 4, &bm));

  // forward: layer l consumes the dense activation of layer l-1 (kept only
  // until then) and leaves the packed sample of its own output for layer l+1
  RAD_TRY(model_clear_max_seg(c, m));
  const bool proj = m->scheme == RAD_PROJECT_SHARED || m->scheme == RAD_PROJECT_PER_EXAMPLE;
  rad_sampling s0 = *sm;
  if (!proj) {
    RAD_TRY(store_plan(c, m->stores[0], &s0, static_cast<uint32_t*>(bm), false));
    RAD_TRY(store_pack(c, m->stores[0], x, 0));
  }
  const void* a_in = x;
  for (int l = 0; l < Lc; ++l) {
    const bool last = l == Lc - 1;
    StoreView nv; const StoreView* next = nullptr;
    if (proj) {          // the layer input is projected by a GEMM of its own; nothing is fused into the epilogue
      rad_sampling sl = *sm; sl.stream_id = sm->stream_id + (uint32_t)l;
      RAD_TRY(project_forward(c, m->stores[(size_t)l], &sl, a_in));
    } else if (!last) {
      rad_store* sn = m->stores[(size_t)l + 1];
      if (sn->scheme != RAD_EXACT) {
        rad_sampling sl = *sm; sl.stream_id = sm->stream_id + (uint32_t)(l + 1);
        RAD_TRY(store_plan(c, sn, &sl, static_cast<uint32_t*>(bm), false));
        nv = store_view(sn, 0); next = &nv;
      }
    }
    // The epilogue packs with one thread per tile row, which walks the row's kept columns one by one: fine
    // for a few dozen per 256 columns, slow for denser samples.  Large layers run one 256x256 workgroup per
    // CU in a single wave of workgroups, so nothing overlaps that walk; there a dense sample is packed by the
    // pack kernel afterwards, which re-reads y at full occupancy (measured equal at a kept fraction of 0.1).
    const bool pack_after = next != nullptr && m->dtype == kBF16 && m->stores[(size_t)l + 1]->p > 0.125 &&
                            (int64_t)B * m->dims[(size_t)l + 1] >= (int64_t(1) << 22);
    if (pack_after) next = nullptr;
    void* y = last ? m->logits : (m->stores[(size_t)l + 1]->scheme == RAD_EXACT ? m->stores[(size_t)l + 1]->values
                                                                                 : m->act[l & 1]);
    rad_store* s = m->stores[(size_t)l];
    RAD_TRY(forward_gemm(c, m->dtype, B, (int)m->dims[(size_t)l + 1], (int)m->dims[(size_t)l], a_in, m->dims[(size_t)l],
                         Wp(l), bp(l), !last, y, s->bits, s->bits_pitch, next, nullptr, 0, 0, nullptr));
    if (pack_after) RAD_TRY(store_pack(c, m->stores[(size_t)l + 1], y, 0));
    a_in = y;
  }
  RAD_TRY(softmax_call(c, m->logits, labels, B, (int)m->dims[(size_t)Lc], m->dtype, m->dyb[0], loss_host ? c->loss_dev : nullptr,
                       m->last_pitch));

  // backward from the stores.  dyb holds g = dL/dh of the layer at hand: the loss gradient for the last
  // layer (no ReLU), and below it the dX of the layer above, masked by this layer's ReLU bits in that
  // GEMM's epilogue.
  int cur = 0;
  for (int l = Lc - 1; l >= 0; --l) {
    rad_store* s = m->stores[(size_t)l];
    const int N = (int)m->dims[(size_t)l + 1], D = (int)m->dims[(size_t)l];
    const int g_ld = (l == Lc - 1 && m->last_pitch) ? m->last_pitch : 0;      // row pitch of this layer's g, if padded
    RAD_TRY(dW_gemm(c, s, 0, m->dyb[cur], N, nullptr, 0, static_cast<float*>(grads[l * per]), 0, 1, g_ld));
    if (m->has_bias)
      RAD_TRY(colsum_call(c, m->dyb[cur], m->dtype, B, N, nullptr, 0, nullptr, 0, 0,
                          static_cast<float*>(grads[l * per + 1]), nullptr, 0, 0, 0, g_ld));
    if (l > 0) {
      rad_store* below = m->stores[(size_t)l - 1];
      RAD_TRY(dX_gemm(c, m->dtype, B, D, N, m->dyb[cur], nullptr, 0, Wp(l), m->dyb[cur ^ 1], below->bits,
                      below->bits_pitch, g_ld));
      cur ^= 1;
    }
  }
  return step_finish(c, m, loss_host);
}

extern "C" rad_status rad_model_create_rnn(rad_ctx* c, int64_t batch, int64_t T, int64_t d_input, int64_t hidden,
                                           int64_t classes, int32_t scheme, double p, rad_model** out) {
  if (!c) return RAD_ERR_NULL;
  if (!out) return fail(c, RAD_ERR_NULL, "out is null");
  *out = nullptr;
  RAD_TRY(check_scheme(c, scheme, p));
  if (batch < 1 || T < 1 || d_input < 1 || hidden < 1 || classes < 1) return fail(c, RAD_ERR_SHAPE, "bad RNN shape");
  if (d_input > 8) return fail(c, RAD_ERR_UNSUPPORTED, "RNN input width above 8");
  if (T > (1 << 20)) return fail(c, RAD_ERR_SHAPE, "T above 2^20");
  rad_model* m = new rad_model();
  m->kind = kRnn; m->dtype = kF32; m->scheme = scheme; m->p = p; m->batch = batch;
  m->T = T; m->d_input = d_input; m->hidden = hidden; m->classes = classes;
  rad_layer L; std::memset(&L, 0, sizeof(L));
  L.kind = RAD_LINEAR; L.dtype = RAD_F32; L.batch = batch; L.d_in = hidden; L.d_out = hidden; L.relu = 0;
  rad_store* s = nullptr;
  rad_status st = rad_store_create(c, &L, scheme, p, (int32_t)(T > 1 ? T - 1 : 1), &s);
  if (st != RAD_OK) { rad_model_destroy(m); return st; }
  m->stores.push_back(s);
  L.d_out = classes;
  st = rad_store_create(c, &L, scheme, p, 1, &s);
  if (st != RAD_OK) { rad_model_destroy(m); return st; }
  m->stores.push_back(s);
  const size_t hb = (size_t)batch * hidden * 4;
  bool ok = true;
  for (void** p2 : {&m->act[0], &m->act[1], &m->dyb[0], &m->dyb[1]}) ok = ok && hipMalloc(p2, hb) == hipSuccess;
  ok = ok && hipMalloc(&m->logits, (size_t)batch * classes * 4) == hipSuccess;
  ok = ok && hipMalloc((void**)&m->rnn_bits, (size_t)T * batch * ((hidden + 31) / 32) * 4) == hipSuccess;
  ok = ok && hipMalloc((void**)&m->rnn_g, (size_t)2 * kRnnChunk * hb) == hipSuccess;
  const size_t bmw = m->stores[0]->bitmap_words() + m->stores[1]->bitmap_words();
  if (bmw) ok = ok && hipMalloc((void**)&m->bitmap_ws, bmw * 4) == hipSuccess;
  if (!ok) { rad_model_destroy(m); return fail(c, RAD_ERR_DEVICE, "model allocation failed"); }
  { rad_status fs = model_share_flags(c, m); if (fs != RAD_OK) { rad_model_destroy(m); return fs; } }
  *out = m;
  return RAD_OK;
}

// BPTT over the unrolled ReLU RNN of Appendix A.  params/grads order:
// W_ih, W_hh, b, W_ho, b_o.
static rad_status rnn_step(rad_ctx* c, rad_model* m, const rad_sampling* sm, const void* x, const int32_t* labels,
                           void* const* params, void* const* grads, float* loss_host) {
  for (int i = 0; i < 5; ++i)
    if (!params[i] || !grads[i]) return fail(c, RAD_ERR_NULL, "null parameter or gradient pointer");
  const int B = (int)m->batch, H = (int)m->hidden, T = (int)m->T, I = (int)m->d_input, C = (int)m->classes;
  const float* W_ih = static_cast<const float*>(params[0]);
  const float* W_hh = static_cast<const float*>(params[1]);
  const float* b = static_cast<const float*>(params[2]);
  const float* W_ho = static_cast<const float*>(params[3]);
  const float* b_o = static_cast<const float*>(params[4]);
  float* dW_ih = static_cast<float*>(grads[0]);
  float* dW_hh = static_cast<float*>(grads[1]);
  float* db = static_cast<float*>(grads[2]);
  float* dW_ho = static_cast<float*>(grads[3]);
  float* db_o = static_cast<float*>(grads[4]);
  const float* xs = static_cast<const float*>(x);
  rad_store* s_hh = m->stores[0];
  rad_store* s_ho = m->stores[1];
  const int bp = (H + 31) / 32;

  // all keep sets of the step up front: they depend on (seed, step) only
  RAD_TRY(model_clear_max_seg(c, m));
  if (T > 1) {
    rad_sampling s1 = *sm; s1.step = sm->step + 2;      // slot s holds h_{s+1}, drawn with step = s+2
    RAD_TRY(store_plan(c, s_hh, &s1, m->bitmap_ws, false));
  }
  rad_sampling s2 = *sm; s2.stream_id = sm->stream_id + 1; s2.step = 0;
  RAD_TRY(store_plan(c, s_ho, &s2, m->bitmap_ws ? m->bitmap_ws + s_hh->bitmap_words() : nullptr, false));

  // forward: h_t = ReLU(x_t W_ih + h_{t-1} W_hh + b); h_0 = 0 so step 1 has no contraction.
  // Stores whose rows are planned one by one take the samples of h_1 .. h_{T-1} eight steps at a time: the steps'
  // outputs go to a ring of eight row blocks (the chunk buffer of the backward pass, idle now) and one pack launch
  // covers their consecutive store slots.
  const bool chunk_pack = T > 1 && (s_hh->scheme == RAD_BERNOULLI || s_hh->scheme == RAD_FIXEDK_PER_EXAMPLE ||
                                    s_hh->scheme == RAD_REPLACE_PER_EXAMPLE);
  auto ring = [&](int t) -> float* { return m->rnn_g + (size_t)((t - 1) % kRnnChunk) * B * H; };     // h_t, t < T
  for (int t = 1; t <= T; ++t) {
    StoreView nv; const StoreView* next = nullptr;
    rad_store* target = t < T ? s_hh : s_ho;
    void* y = m->act[t & 1];
    if (target->scheme == RAD_EXACT) {
      y = static_cast<char*>(target->values) + (t < T ? (size_t)(t - 1) * B * H * 4 : 0);
    } else if (target->project()) {
      // the projection of h_t is a GEMM of its own after the step (Appendix A, RNN details: "project")
    } else if (t < T && chunk_pack) {
      y = ring(t);
    } else { nv = store_view(target, t < T ? t - 1 : 0); next = &nv; }
    const void* hin = t == 1 ? m->act[0] : (s_hh->scheme == RAD_EXACT
                          ? static_cast<const void*>(static_cast<char*>(s_hh->values) + (size_t)(t - 2) * B * H * 4)
                          : chunk_pack ? static_cast<const void*>(ring(t - 1)) : m->act[(t - 1) & 1]);
    RAD_TRY(forward_gemm(c, kF32, B, H, t == 1 ? 0 : H, hin, H, W_hh, b, 1, y, m->rnn_bits + (size_t)(t - 1) * B * bp,
                         bp, next, xs + (size_t)(t - 1) * I, (int64_t)T * I, I, W_ih));
    if (target->project()) {
      rad_sampling sp = t < T ? *sm : s2;
      if (t < T) sp.step = sm->step + (uint32_t)t + 1;      // slot t - 1 holds h_t, drawn with step = t + 1
      RAD_TRY(project_forward(c, target, &sp, y, t < T ? t - 1 : 0));
    }
    if (t < T && chunk_pack && (t % kRnnChunk == 0 || t == T - 1)) {
      const int t0 = (t - 1) / kRnnChunk * kRnnChunk + 1;          // first step of the chunk; its output is ring block 0
      StoreView v = store_view(s_hh, t0 - 1);
      v.rows = (t - t0 + 1) * B;
      HIP_TRY(c, timed(c, "pack_f32", [&](const char**) { return launch_pack(ring(t0), kF32, v, c->stream); }));
    }
  }
  const void* hT = s_ho->scheme == RAD_EXACT ? s_ho->values : m->act[T & 1];
  RAD_TRY(forward_gemm(c, kF32, B, C, H, hT, H, W_ho, b_o, 0, m->logits, nullptr, 0, nullptr, nullptr, 0, 0, nullptr));
  RAD_TRY(softmax_call(c, m->logits, labels, B, C, kF32, m->dyb[0], loss_host ? c->loss_dev : nullptr));

  // backward
  float* dz = static_cast<float*>(m->dyb[0]);
  RAD_TRY(dW_gemm(c, s_ho, 0, dz, C, nullptr, 0, dW_ho, 0));
  RAD_TRY(colsum_call(c, dz, kF32, B, C, nullptr, 0, nullptr, 0, 0, db_o, nullptr, 0));
  // dyb holds g_t = dL/dh_t masked by the ReLU bits of step t (applied in the epilogue of the GEMM that
  // produces it)
  // g_t, t >= 2, goes to row block (t - 2) % G of rnn_g; steps 2 + jG .. 1 + (j + 1)G share a chunk, whose store
  // slots t - 2 are consecutive, so that dW_hh of the chunk is one contraction over (steps x batch) rows instead
  // of one short contraction per step.  Stores planned per step (shared index sets) or rebuilt before use
  // (index-free) keep the step-by-step form (two row blocks, used in turn).  g_1 has no dW_hh and lives in dyb[1].
  const bool per_row = s_hh->scheme == RAD_EXACT || s_hh->scheme == RAD_BERNOULLI || s_hh->scheme == RAD_FIXEDK_PER_EXAMPLE ||
                       s_hh->scheme == RAD_REPLACE_PER_EXAMPLE;
  const int G = per_row ? kRnnChunk : 1;
  const int Gp = G > 1 ? 2 * G : 2;                      // row blocks in use: two chunks, or two single steps
  const size_t gstride = (size_t)B * H;
  auto g_of = [&](int t) -> float* { return t >= 2 ? m->rnn_g + (size_t)((t - 2) % Gp) * gstride : static_cast<float*>(m->dyb[1]); };
  // With chunks, their gradients (dW_hh, db, dW_ih: nothing downstream waits for them) are enqueued on a side
  // stream while the main stream goes on with the chain of dX GEMMs into the other chunk's rows; the main stream
  // waits before it writes into a chunk whose last reader may still be running, and at the end.
  bool side = G > 1 && !(c->timing && c->filter.empty());
  if (side && !c->side) {
    bool ok = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) == hipSuccess;
    for (hipEvent_t* e : {&c->ev_ready[0], &c->ev_ready[1], &c->ev_done[0], &c->ev_done[1], &c->ev_join})
      ok = ok && hipEventCreateWithFlags(e, hipEventDisableTiming) == hipSuccess;
    if (!ok) return fail(c, RAD_ERR_DEVICE, "side stream");
  }
  bool done_pending[2] = {false, false};
  RAD_TRY(dX_gemm(c, kF32, B, H, C, dz, nullptr, 0, W_ho, g_of(T), m->rnn_bits + (size_t)(T - 1) * B * bp, bp));
  if (T == 1) HIP_TRY(c, launch_fill_u32(reinterpret_cast<uint32_t*>(dW_hh), 0u, (int64_t)H * H, c->stream));
  bool first_dw = true, first_cs = true;
  rad_status rs = RAD_OK;
  // a failing call inside the loop records its status and leaves through the join below, never past it
  auto ok = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && rs == RAD_OK) rs = hip_fail(c, e, what);
    return rs == RAD_OK;
  };
  for (int t = T; t >= 1 && rs == RAD_OK; --t) {
    if (t >= 2 && (t - 2) % G == 0) {                     // g of the whole chunk t .. t_hi is there
      const int n = std::min(T, t + G - 1) - t + 1;
      const int half = ((t - 2) / G) & 1;
      if (side) {
        if (!ok(hipEventRecord(c->ev_ready[half], c->stream), "event record")) break;
        if (!ok(hipStreamWaitEvent(c->side, c->ev_ready[half], 0), "stream wait")) break;
        std::swap(c->stream, c->side);
      }
      rs = dW_gemm(c, s_hh, t - 2, g_of(t), H, nullptr, 0, dW_hh, first_dw ? 0 : 1, n);
      first_dw = false;
      // db and dW_ih of the chunk: rows in blocks of B per step, step q weighing with x_{t+q}
      if (rs == RAD_OK)
        rs = colsum_call(c, g_of(t), kF32, n * B, H, nullptr, 0, xs + (size_t)(t - 1) * I, (int64_t)T * I, I, db,
                         dW_ih, first_cs ? 0 : 1, B, I);
      first_cs = false;
      if (side) {
        std::swap(c->stream, c->side);
        if (rs == RAD_OK && ok(hipEventRecord(c->ev_done[half], c->side), "event record")) done_pending[half] = true;
        // the dX below starts the other chunk's rows: their last reader must be through
        if (rs == RAD_OK && done_pending[half ^ 1]) {
          if (ok(hipStreamWaitEvent(c->stream, c->ev_done[half ^ 1], 0), "stream wait")) done_pending[half ^ 1] = false;
        }
      }
      if (rs != RAD_OK) break;
    }
    if (t == 1) {
      if (side) {                                         // db and dW_ih accumulate in stream order: join first
        if (!ok(hipEventRecord(c->ev_join, c->side), "event record")) break;
        if (!ok(hipStreamWaitEvent(c->stream, c->ev_join, 0), "stream wait")) break;
        side = false;
      }
      rs = colsum_call(c, g_of(1), kF32, B, H, nullptr, 0, xs, (int64_t)T * I, I, db, dW_ih, first_cs ? 0 : 1);
      first_cs = false;
    }
    if (t >= 2 && rs == RAD_OK)
      rs = dX_gemm(c, kF32, B, H, H, g_of(t), nullptr, 0, W_hh, g_of(t - 1),
                   m->rnn_bits + (size_t)(t - 2) * B * bp, bp);
  }
  if (c->side && G > 1) {                                 // whatever happened, the main stream ends behind the side stream
    (void)hipEventRecord(c->ev_join, c->side);
    (void)hipStreamWaitEvent(c->stream, c->ev_join, 0);
  }
  RAD_TRY(rs);
  return step_finish(c, m, loss_host);
}

extern "C" rad_status rad_model_create_cnn(rad_ctx* c, int64_t batch, int32_t n_conv, const int32_t* channels,
                                           const int32_t* pool, int32_t ksize, int32_t height, int32_t width,
                                           int32_t classes, int32_t scheme, double p, rad_model** out) {
  if (!c) return RAD_ERR_NULL;
  if (!out || !channels || !pool) return fail(c, RAD_ERR_NULL, "null argument");
  *out = nullptr;
  RAD_TRY(check_scheme(c, scheme, p));
  if (n_conv < 1 || n_conv > 32 || batch < 1 || classes < 1 || ksize < 1 || (ksize & 1) == 0)
    return fail(c, RAD_ERR_SHAPE, "bad CNN shape (odd kernel size, at least one conv)");
  if (scheme == RAD_PROJECT_SHARED || scheme == RAD_PROJECT_PER_EXAMPLE) return fail(c, RAD_ERR_UNSUPPORTED, "the projection schemes serve MLP models only");
  for (int l = 0; l < n_conv; ++l)
    if (pool[l] < 0 || pool[l] > 2) return fail(c, RAD_ERR_PARAM, "pool[l] is 0 (none), 1 (max) or 2 (average)");
  rad_model* m = new rad_model();
  m->kind = kCnn; m->dtype = kF32; m->scheme = scheme; m->p = p; m->batch = batch; m->ksize = ksize;
  m->classes = classes; m->has_bias = 1;
  int h = height, w = width;
  size_t widest = (size_t)channels[0] * h * w;
  for (int l = 0; l < n_conv; ++l) {
    if (channels[l] < 1 || channels[l + 1] < 1 || h < 1 || w < 1 || (h * w) % 64 != 0 || channels[l + 1] > 64) {
      rad_model_destroy(m);
      return fail(c, RAD_ERR_UNSUPPORTED, "conv layers need H*W a multiple of 64 and at most 64 output channels");
    }
    rad_layer L; std::memset(&L, 0, sizeof(L));
    L.kind = RAD_CONV2D; L.dtype = RAD_F32; L.batch = batch;
    L.c_in = channels[l]; L.c_out = channels[l + 1]; L.h = h; L.w = w; L.kh = L.kw = ksize; L.pad = (ksize - 1) / 2;
    L.d_in = (int64_t)L.c_in * h * w; L.d_out = (int64_t)L.c_out * h * w; L.relu = 1; L.has_bias = 1;
    rad_store* s = nullptr;
    rad_status st = rad_store_create(c, &L, scheme, p, 1, &s);
    if (st != RAD_OK) { rad_model_destroy(m); return st; }
    m->stores.push_back(s);
    rad_model::Conv cv{channels[l], channels[l + 1], h, w, pool[l], nullptr};
    if ((size_t)L.d_out > widest) widest = (size_t)L.d_out;
    if (cv.pool) {
      if ((h & 1) || (w & 1)) { rad_model_destroy(m); return fail(c, RAD_ERR_SHAPE, "pooled layers need even H and W"); }
      if (cv.pool == 1) {      // max pool keeps 2-bit window positions; the average pool keeps nothing
        const size_t words = ((size_t)batch * cv.co * (h / 2) * (w / 2) + 15) / 16;
        if (hipMalloc((void**)&cv.arg, words * 4) != hipSuccess) { rad_model_destroy(m); return fail(c, RAD_ERR_DEVICE, "model allocation failed"); }
      }
      h /= 2; w /= 2;
    }
    m->convs.push_back(cv);
  }
  m->fc_in = channels[n_conv] * h * w;
  rad_layer L; std::memset(&L, 0, sizeof(L));
  L.kind = RAD_LINEAR; L.dtype = RAD_F32; L.batch = batch; L.d_in = m->fc_in; L.d_out = classes; L.has_bias = 1;
  rad_store* s = nullptr;
  rad_status st = rad_store_create(c, &L, scheme, p, 1, &s);
  if (st != RAD_OK) { rad_model_destroy(m); return st; }
  m->stores.push_back(s);
  bool ok = true;
  for (int i = 0; i < 3; ++i) ok = ok && hipMalloc(&m->buf[i], (size_t)batch * widest * 4) == hipSuccess;
  ok = ok && hipMalloc(&m->logits, (size_t)batch * classes * 4) == hipSuccess;
  ok = ok && hipMalloc(&m->dyb[0], (size_t)batch * classes * 4) == hipSuccess;
  if (!ok) { rad_model_destroy(m); return fail(c, RAD_ERR_DEVICE, "model allocation failed"); }
  { rad_status fs = model_share_flags(c, m); if (fs != RAD_OK) { rad_model_destroy(m); return fs; } }
  *out = m;
  return RAD_OK;
}

// conv as implicit im2col GEMM: y[B,co,h,w] = act(conv(src[B,ci,h,w], W[(ci,k,k)][co]) + bias)
static rad_status conv_gemm(rad_ctx* c, int B, int ci, int co, int h, int w, int ks, const float* src, const float* W,
                            const float* bias, int relu, float* y, uint32_t* bits, int bits_pitch) {
  GemmArgs g = gemm_zero();
  g.M = B * h * w; g.N = co; g.K = ci * ks * ks;
  g.A = src; g.B = W; g.ldb = co;
  g.cv_C = ci; g.cv_H = h; g.cv_W = w; g.cv_KH = ks; g.cv_KW = ks; g.cv_pad = (ks - 1) / 2; g.cv_N = co;
  g.bias = bias; g.relu = relu; g.y = y; g.bits = relu ? bits : nullptr; g.bits_pitch = bits_pitch;
  // the patch-staged kernel where it serves the shape, else the general im2col GEMM
  bool served = true;
  HIP_TRY(c, timed(c, "conv_fwd_direct", [&](const char**) {
    const hipError_t e = launch_conv_fwd_direct(g, c->stream);
    if (e == hipErrorInvalidValue) { served = false; return hipSuccess; }
    return e;
  }));
  if (served) return RAD_OK;
  return run_gemm_call(c, kF32, kOpIm2colRows, kOpMN, kEpiConv, g);
}

// what the convolution kernels serve: fp32, square odd kernels, at most 64 output channels (one tile column),
// H*W a multiple of the 64-row tile (a tile never straddles two images)
static rad_status conv_limits(rad_ctx* c, const rad_layer* L) {
  if (L->kh != L->kw) return fail(c, RAD_ERR_UNSUPPORTED, "conv kernels must be square");
  if (L->c_out > 64 || (L->h * L->w) % 64 != 0 || L->c_in > 64)
    return fail(c, RAD_ERR_UNSUPPORTED, "conv layers need H*W a multiple of 64 and at most 64 input and output channels");
  return RAD_OK;
}

static rad_status conv_masked_dy(rad_ctx* c, const rad_layer* L, const rad_store* s, const void* dy, const float** g) {
  if (!L->relu) { *g = static_cast<const float*>(dy); return RAD_OK; }
  void* buf = nullptr;
  RAD_TRY(ws_get(c, WS_CONVG, (size_t)L->batch * L->d_out * 4, &buf));
  HIP_TRY(c, timed(c, "unpool_mask", [&](const char**) {
    return launch_unpool_mask(static_cast<const float*>(dy), (int)L->batch, L->c_out, L->h, L->w, 0, nullptr, s->bits,
                              s->bits_pitch, static_cast<float*>(buf), c->stream);
  }));
  *g = static_cast<const float*>(buf);
  return RAD_OK;
}

// dW [ci*ks*ks][co] (and dbias [co], if given) of a convolution from the sampled input in `s` and g = dL/dh
// [B][co][h][w] (Figure 5: the sampled x~ is scattered back to a dense transient and contracted with g)
static rad_status conv_dW_call(rad_ctx* c, const rad_store* s, int B, int ci, int co, int h, int w, int ks, const float* g,
                               float* dW, float* dbias) {
  const int HW = h * w;
  const void* xt = s->values;
  if (s->scheme != RAD_EXACT) {
    void* dense = nullptr;
    RAD_TRY(ws_get(c, WS_DENSE, (size_t)B * s->cols * 4, &dense));
    StoreView v;                                   // an index-free store is read through its rebuild
    RAD_TRY(backward_view(c, s, 0, &v));
    HIP_TRY(c, timed(c, "unpack", [&](const char**) { return launch_unpack(v, kF32, dense, c->stream); }));
    xt = dense;
  }
  if (const int splits = conv_dw_direct_splits(B, ci, co, h, w, ks)) {
    const int64_t mn = (int64_t)ci * ks * ks * co;
    void* part = nullptr;
    RAD_TRY(ws_get(c, WS_SPLITK, (size_t)splits * mn * 4, &part));
    HIP_TRY(c, timed(c, "conv_dw_direct", [&](const char**) {
      return launch_conv_dw_direct(static_cast<const float*>(xt), g, static_cast<float*>(part), B, ci, co, h, w, ks, c->stream);
    }));
    HIP_TRY(c, timed(c, "splitk_reduce", [&](const char**) {
      return launch_splitk_reduce(static_cast<const float*>(part), splits, mn, dW, 0, c->stream);
    }));
  } else {
  GemmArgs a = gemm_zero();
  a.M = ci * ks * ks; a.N = co; a.K = B * HW;
  a.A = xt; a.B = g;
  a.cv_C = ci; a.cv_H = h; a.cv_W = w; a.cv_KH = ks; a.cv_KW = ks; a.cv_pad = (ks - 1) / 2; a.cv_N = co;
  a.k_split = 1024; a.k_splits = (a.K + a.k_split - 1) / a.k_split;
  void* part = nullptr;
  RAD_TRY(ws_get(c, WS_SPLITK, (size_t)a.k_splits * a.M * a.N * 4, &part));
  a.C = part; a.ldc = a.N;
  RAD_TRY(run_gemm_call(c, kF32, kOpIm2colK, kOpKBatched, kEpiSplitK, a));
  HIP_TRY(c, timed(c, "splitk_reduce", [&](const char**) {
    return launch_splitk_reduce(static_cast<const float*>(part), a.k_splits, (int64_t)a.M * a.N, dW, 0, c->stream);
  }));
  }
  if (dbias) {
    const int cs_splits = B < 32 ? B : 32;
    void* cs_part = nullptr;
    RAD_TRY(ws_get(c, WS_COLSUM, (size_t)co * cs_splits * 4, &cs_part));
    HIP_TRY(c, timed(c, "channel_sum", [&](const char**) {
      return launch_channel_sum(g, B, co, HW, dbias, static_cast<float*>(cs_part), cs_splits, c->stream);
    }));
  }
  return RAD_OK;
}

// dX [B][ci][h][w] = the transposed convolution of g with W, exact (never sampled)
static rad_status conv_dX_call(rad_ctx* c, int B, int ci, int co, int h, int w, int ks, const float* g, const float* W,
                               float* dX) {
  void* wt = nullptr;
  RAD_TRY(ws_get(c, WS_WT, (size_t)co * ks * ks * ci * 4, &wt));
  HIP_TRY(c, timed(c, "flip_weights", [&](const char**) {
    return launch_flip_weights(W, ci, ks, ks, co, static_cast<float*>(wt), c->stream);
  }));
  return conv_gemm(c, B, co, ci, h, w, ks, g, static_cast<const float*>(wt), nullptr, 0, dX, nullptr, 0);
}

// params/grads order: W_0, b_0, ..., W_{n-1}, b_{n-1}, W_fc, b_fc
static rad_status cnn_step(rad_ctx* c, rad_model* m, const rad_sampling* sm, const void* x, const int32_t* labels,
                           void* const* params, void* const* grads, float* loss_host) {
  const int nc = (int)m->convs.size();
  const int B = (int)m->batch, ks = m->ksize, C = (int)m->classes;
  for (int i = 0; i < 2 * (nc + 1); ++i)
    if (!params[i] || !grads[i]) return fail(c, RAD_ERR_NULL, "null parameter or gradient pointer");
  size_t bm_words = 0;
  for (rad_store* s : m->stores) if (s->bitmap_words() > bm_words) bm_words = s->bitmap_words();
  void* bm = nullptr;
  if (bm_words) RAD_TRY(ws_get(c, WS_BITMAP, bm_words * 4, &bm));
  RAD_TRY(model_clear_max_seg(c, m));

  // forward: every conv input is sampled (flattened per example), then convolved exactly
  const float* act = static_cast<const float*>(x);
  int in_buf = -1;                    // buffer index holding `act` (-1: caller's x)
  for (int l = 0; l < nc; ++l) {
    const rad_model::Conv& cv = m->convs[(size_t)l];
    rad_store* s = m->stores[(size_t)l];
    rad_sampling sl = *sm; sl.stream_id = sm->stream_id + (uint32_t)l;
    RAD_TRY(store_plan(c, s, &sl, static_cast<uint32_t*>(bm), false));
    RAD_TRY(store_pack(c, s, act, 0));
    const int yb = (in_buf + 1 + 3) % 3, pb = (in_buf + 2 + 3) % 3;
    RAD_TRY(conv_gemm(c, B, cv.ci, cv.co, cv.h, cv.w, ks, act, static_cast<const float*>(params[2 * l]),
                      static_cast<const float*>(params[2 * l + 1]), 1, static_cast<float*>(m->buf[yb]), s->bits,
                      s->bits_pitch));
    if (cv.pool) {
      if (cv.pool == 1) {
        HIP_TRY(c, timed(c, "maxpool", [&](const char**) {
          return launch_maxpool_fwd(static_cast<const float*>(m->buf[yb]), B * cv.co, cv.h, cv.w,
                                    static_cast<float*>(m->buf[pb]), cv.arg, c->stream);
        }));
      } else {
        HIP_TRY(c, timed(c, "avgpool", [&](const char**) {
          return launch_avgpool_fwd(static_cast<const float*>(m->buf[yb]), B * cv.co, cv.h, cv.w,
                                    static_cast<float*>(m->buf[pb]), c->stream);
        }));
      }
      act = static_cast<const float*>(m->buf[pb]); in_buf = pb;
    } else { act = static_cast<const float*>(m->buf[yb]); in_buf = yb; }
  }
  rad_store* sfc = m->stores[(size_t)nc];
  {
    rad_sampling sl = *sm; sl.stream_id = sm->stream_id + (uint32_t)nc;
    RAD_TRY(store_plan(c, sfc, &sl, static_cast<uint32_t*>(bm), false));
    RAD_TRY(store_pack(c, sfc, act, 0));
  }
  RAD_TRY(forward_gemm(c, kF32, B, C, m->fc_in, act, m->fc_in, params[2 * nc], static_cast<const float*>(params[2 * nc + 1]),
                       0, m->logits, nullptr, 0, nullptr, nullptr, 0, 0, nullptr));
  RAD_TRY(softmax_call(c, m->logits, labels, B, C, kF32, m->dyb[0], loss_host ? c->loss_dev : nullptr));

  // backward
  RAD_TRY(dW_gemm(c, sfc, 0, m->dyb[0], C, nullptr, 0, static_cast<float*>(grads[2 * nc]), 0));
  RAD_TRY(colsum_call(c, m->dyb[0], kF32, B, C, nullptr, 0, nullptr, 0, 0, static_cast<float*>(grads[2 * nc + 1]),
                      nullptr, 0));
  int db_ = (in_buf + 1) % 3;          // upstream gradient buffer; the forward activations are dead by now
  RAD_TRY(dX_gemm(c, kF32, B, m->fc_in, C, m->dyb[0], nullptr, 0, params[2 * nc], m->buf[db_]));
  for (int l = nc - 1; l >= 0; --l) {
    const rad_model::Conv& cv = m->convs[(size_t)l];
    rad_store* s = m->stores[(size_t)l];
    const int gb = (db_ + 1) % 3, nb_ = (db_ + 2) % 3;
    float* g = static_cast<float*>(m->buf[gb]);
    // g = dL/dh of this layer: route through the pool, then the 1-bit ReLU Jacobian (Section 4.2)
    HIP_TRY(c, timed(c, "unpool_mask", [&](const char**) {
      return launch_unpool_mask(static_cast<const float*>(m->buf[db_]), B, cv.co, cv.h, cv.w, cv.pool, cv.arg, s->bits,
                                s->bits_pitch, g, c->stream);
    }));
    RAD_TRY(conv_dW_call(c, s, B, cv.ci, cv.co, cv.h, cv.w, ks, g, static_cast<float*>(grads[2 * l]),
                         static_cast<float*>(grads[2 * l + 1])));
    if (l > 0) {
      RAD_TRY(conv_dX_call(c, B, cv.ci, cv.co, cv.h, cv.w, ks, g, static_cast<const float*>(params[2 * l]),
                           static_cast<float*>(m->buf[nb_])));
      db_ = nb_;
    }
  }
  return step_finish(c, m, loss_host);
}

extern "C" rad_status rad_train_step(rad_ctx* c, rad_model* m, const rad_sampling* sm, const void* x,
                                     const int32_t* labels, void* const* params, void* const* grads,
                                     float* loss_host) {
  if (!c) return RAD_ERR_NULL;
  if (!m || !sm || !x || !labels || !params || !grads) return fail(c, RAD_ERR_NULL, "null argument");
  RAD_TRY(check_scheme(c, sm->scheme, sm->p));
  if (sm->scheme != m->scheme || sm->p != m->p) return fail(c, RAD_ERR_PARAM, "sampling does not match the model");
  if (m->kind == kMlp) return mlp_step(c, m, sm, x, labels, params, grads, loss_host);
  if (m->kind == kRnn) return rnn_step(c, m, sm, x, labels, params, grads, loss_host);
  return cnn_step(c, m, sm, x, labels, params, grads, loss_host);
}

