// Host side of the GAC step library: context, planner, pointer-table upload, C ABI.
// Interface and semantics: include/gac.h.  Kernels: gac_kernels.hip.

#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "gac_internal.h"

using gac::AdamScalars;
using gac::AdamSeg;
using gac::DecideParams;
using gac::Seg;

namespace {

constexpr int kPinnedSlots = 4;         // ring of pinned staging tables for pointer uploads
constexpr int kChunkMultiple = 2048;    // chunk_elems granularity (256 threads x 8 elements)
constexpr int kMaxProfiledSteps = 1024;

int64_t elem_size(int dtype) { return dtype == GAC_BF16 ? 2 : 4; }

int default_chunk_elems(int dtype) { return gac::kDefaultChunkBytes / static_cast<int>(elem_size(dtype)); }

bool thresholds_ok(double c_low, double c_high) {
  // Section 4.2: 0 < c_low < c_high.  (NaN fails every comparison.)
  return c_low > 0.0 && c_high > c_low && std::isfinite(c_low) && !std::isnan(c_high);
}

// Cuts the tensor list into chunks.  first_chunk gets n_tensors + 1 entries.
int plan(const int64_t* numel, int32_t n_tensors, int chunk_elems, std::vector<int64_t>* first_chunk,
         int64_t* total) {
  first_chunk->assign(static_cast<size_t>(n_tensors) + 1, 0);
  int64_t c = 0, n = 0;
  for (int32_t j = 0; j < n_tensors; ++j) {
    if (numel[j] < 0) return GAC_ERR_INVALID_ARG;
    (*first_chunk)[j] = c;
    c += (numel[j] + chunk_elems - 1) / chunk_elems;
    n += numel[j];
  }
  (*first_chunk)[n_tensors] = c;
  *total = n;
  return GAC_OK;
}

int resolve_chunk_elems(int dtype, int chunk_elems, int* out) {
  if (dtype != GAC_F32 && dtype != GAC_BF16) return GAC_ERR_INVALID_ARG;
  if (chunk_elems == 0) chunk_elems = default_chunk_elems(dtype);
  if (chunk_elems < 0 || chunk_elems % kChunkMultiple != 0) return GAC_ERR_INVALID_ARG;
  *out = chunk_elems;
  return GAC_OK;
}

struct StepEvents {
  hipEvent_t e[4];  // before reduce, after reduce, after finalize, after apply
};

}  // namespace

struct gac_ctx {
  int device = 0;
  int dtype = GAC_BF16;
  int n_tensors = 0;
  std::vector<int64_t> numel;
  std::vector<int64_t> first_chunk;
  int64_t n_chunks = 0;
  int64_t total = 0;
  int chunk_elems = 0;
  int grid = 1;        // workgroups of the reduce kernel (= number of partials)
  int grid_state = 1;  // workgroups of the state maintenance kernel
  int grid_apply = 1;  // workgroups of the apply kernel
  int grid_adamw = 1;  // workgroups of the fused AdamW apply kernel
  bool apply_blocks_fixed = false;  // gac_config.apply_blocks was given: never re-tuned
  int cus = 1;
  double c_low = 0, c_high = 0, eps = 0, beta = 1;
  double max_grad_norm = 0;
  int64_t* dev_step = nullptr;  // the step counter lives on the device (see DecideParams)

  // record of (c_t, regime) per step: a ring on the device, written by the finalize step
  double* hist_c = nullptr;
  int32_t* hist_regime = nullptr;
  int hist_cap = 0;
  int64_t hist_first = 1;  // earliest step number whose record is valid (moves on reset / import)
  gac_diag* dev_diag = nullptr;
  gac_diag* pinned_diag = nullptr;
  gac_diag* pinned_diag_dev = nullptr;
  int32_t* pinned_sweep = nullptr;      // GAC_MAX_SWEEP_PAIRS x 3 counts, host-mapped
  int32_t* pinned_sweep_dev = nullptr;

  std::vector<void*> state;    // device pointers of d, one per tensor
  void* state_alloc = nullptr; // owned allocation backing `state`, or null
  bool state_is_callers = false;  // the state buffers were provided by the caller

  // Snapshot form (GAC_FLAG_SNAPSHOT_IN_REDUCE): a second state block with the same slicing,
  // snap_delta bytes from the first; *dev_cur says which of the two is the reference state.
  bool snapshot = false;
  void* state1_alloc = nullptr;
  std::vector<void*> state1;
  int64_t snap_delta = 0;
  int32_t* dev_cur = nullptr;
  gac::SnapBuffers snap_buf = {};  // working memory of its pass 1 (one allocation: snap_alloc)
  void* snap_alloc = nullptr;
  int grid_snap = 1;

  // pointer tables
  Seg* dev_segs = nullptr;        // (gradient, state) per tensor: the table the step kernels read
  Seg* dev_segs_state = nullptr;  // (source, destination) of state copies / zeroing: kept apart so
                                  // that an export or import between two replays of a captured
                                  // graph of steps cannot change what that graph reads
  AdamSeg* dev_adam = nullptr;
  Seg* pinned_segs[kPinnedSlots] = {};
  AdamSeg* pinned_adam[kPinnedSlots] = {};
  hipEvent_t slot_event[kPinnedSlots] = {};
  int slot = 0;
  std::vector<const void*> cached_a;  // what dev_segs currently holds in Seg::a
  std::vector<void*> cached_b;        // ... and in Seg::b
  bool segs_valid = false;
  std::vector<AdamSeg> cached_adam;
  bool adam_valid = false;

  double* dev_partials = nullptr;  // 3 doubles per workgroup
  unsigned int* dev_ticket = nullptr;  // arrival counter of the reduction's workgroups (zero between launches)
  unsigned long long* dev_work = nullptr;  // chunk counter of pass 2 (zeroed by the finalize step)
  double* dev_sums = nullptr;      // 3 doubles
  gac_result* dev_result = nullptr;
  gac_result* pinned_result = nullptr;      // host address of the pinned result record
  gac_result* pinned_result_dev = nullptr;  // the same memory as the device addresses it
  hipEvent_t result_event = nullptr;

  bool profiling = false;
  std::vector<StepEvents> prof_pool;
  size_t prof_used = 0;

  std::string hip_err;
};

namespace {

struct DeviceGuard {
  int prev = -1;
  bool changed = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) == hipSuccess && prev != dev) changed = hipSetDevice(dev) == hipSuccess;
  }
  ~DeviceGuard() {
    if (changed) (void)hipSetDevice(prev);
  }
};

// Text of the last HIP failure of any context on this thread; survives a failed gac_init,
// whose context is gone by the time the caller can ask.
thread_local std::string g_last_hip_error;

int fail_hip(gac_ctx* ctx, hipError_t e, const char* what) {
  g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  if (ctx != nullptr) ctx->hip_err = g_last_hip_error;
  return GAC_ERR_HIP;
}

#define GAC_HIP(ctx, call)                                  \
  do {                                                      \
    hipError_t e_ = (call);                                 \
    if (e_ != hipSuccess) return fail_hip(ctx, e_, #call);  \
  } while (0)

// Makes dev_segs hold (a[j], b[j]) for every tensor.  Uploads only when something changed.
int upload_segs(gac_ctx* ctx, const void* const* a, void* const* b, hipStream_t stream) {
  const int n = ctx->n_tensors;
  bool same = ctx->segs_valid;
  for (int j = 0; same && j < n; ++j) same = ctx->cached_a[j] == (a ? a[j] : nullptr) && ctx->cached_b[j] == b[j];
  if (same) return GAC_OK;
  const int s = ctx->slot;
  ctx->slot = (s + 1) % kPinnedSlots;
  GAC_HIP(ctx, hipEventSynchronize(ctx->slot_event[s]));  // the slot's previous upload is done
  Seg* host = ctx->pinned_segs[s];
  for (int j = 0; j < n; ++j) {
    host[j].a = a ? a[j] : nullptr;
    host[j].b = b[j];
    host[j].numel = ctx->numel[j];
    host[j].first_chunk = ctx->first_chunk[j];
    ctx->cached_a[j] = host[j].a;
    ctx->cached_b[j] = host[j].b;
  }
  host[n].a = nullptr;
  host[n].b = nullptr;
  host[n].numel = 0;
  host[n].first_chunk = ctx->n_chunks;
  ctx->segs_valid = false;
  GAC_HIP(ctx, hipMemcpyAsync(ctx->dev_segs, host, sizeof(Seg) * (n + 1), hipMemcpyHostToDevice, stream));
  GAC_HIP(ctx, hipEventRecord(ctx->slot_event[s], stream));
  ctx->segs_valid = true;
  return GAC_OK;
}

// The table of a state operation (zero / copy); rare, so always uploaded.
int upload_state_segs(gac_ctx* ctx, const void* const* a, void* const* b, hipStream_t stream) {
  const int n = ctx->n_tensors;
  const int s = ctx->slot;
  ctx->slot = (s + 1) % kPinnedSlots;
  GAC_HIP(ctx, hipEventSynchronize(ctx->slot_event[s]));
  Seg* host = ctx->pinned_segs[s];
  for (int j = 0; j <= n; ++j) {
    host[j].a = (a && j < n) ? a[j] : nullptr;
    host[j].b = j < n ? b[j] : nullptr;
    host[j].numel = j < n ? ctx->numel[j] : 0;
    host[j].first_chunk = ctx->first_chunk[j];
  }
  GAC_HIP(ctx, hipMemcpyAsync(ctx->dev_segs_state, host, sizeof(Seg) * (n + 1), hipMemcpyHostToDevice, stream));
  GAC_HIP(ctx, hipEventRecord(ctx->slot_event[s], stream));
  return GAC_OK;
}

int upload_adam(gac_ctx* ctx, float* const* p, float* const* m, float* const* v, void* const* pl,
                hipStream_t stream) {
  const int n = ctx->n_tensors;
  bool same = ctx->adam_valid;
  for (int j = 0; same && j < n; ++j) {
    const AdamSeg& c = ctx->cached_adam[j];
    same = c.p == p[j] && c.m == m[j] && c.v == v[j] && c.p_lowp == (pl ? pl[j] : nullptr);
  }
  if (same) return GAC_OK;
  const int s = ctx->slot;
  ctx->slot = (s + 1) % kPinnedSlots;
  GAC_HIP(ctx, hipEventSynchronize(ctx->slot_event[s]));
  AdamSeg* host = ctx->pinned_adam[s];
  for (int j = 0; j < n; ++j) {
    host[j].p = p[j];
    host[j].m = m[j];
    host[j].v = v[j];
    host[j].p_lowp = pl ? pl[j] : nullptr;
    ctx->cached_adam[j] = host[j];
  }
  ctx->adam_valid = false;
  GAC_HIP(ctx, hipMemcpyAsync(ctx->dev_adam, host, sizeof(AdamSeg) * n, hipMemcpyHostToDevice, stream));
  GAC_HIP(ctx, hipEventRecord(ctx->slot_event[s], stream));
  ctx->adam_valid = true;
  return GAC_OK;
}

int check_ptrs(const gac_ctx* ctx, const void* const* ptrs) {
  if (ptrs == nullptr && ctx->n_tensors > 0) return GAC_ERR_INVALID_ARG;
  for (int j = 0; j < ctx->n_tensors; ++j) {
    if (ctx->numel[j] > 0 && ptrs[j] == nullptr) return GAC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(ptrs[j]) % static_cast<uintptr_t>(elem_size(ctx->dtype)) != 0)
      return GAC_ERR_INVALID_ARG;
  }
  return GAC_OK;
}

// In place the gradient and the reference state are read and written by the same pass, so a
// gradient buffer that IS the state buffer cannot work; partial overlaps are the caller's to avoid.
int check_not_state(const gac_ctx* ctx, void* const* grad_ptrs) {
  for (int j = 0; j < ctx->n_tensors; ++j) {
    if (ctx->numel[j] > 0 && grad_ptrs[j] == ctx->state[j]) return GAC_ERR_INVALID_ARG;
    if (ctx->snapshot && ctx->numel[j] > 0 && grad_ptrs[j] == ctx->state1[j]) return GAC_ERR_INVALID_ARG;
  }
  return GAC_OK;
}

// One allocation for the whole state, every tensor's slice 256-byte aligned.
int64_t state_block_bytes(const gac_ctx* ctx) {
  const int64_t es = elem_size(ctx->dtype);
  int64_t bytes = 0;
  for (int j = 0; j < ctx->n_tensors; ++j) bytes += (ctx->numel[j] * es + 255) / 256 * 256;
  return bytes;
}

int alloc_state_block(gac_ctx* ctx, void** alloc, std::vector<void*>* ptrs) {
  const int64_t es = elem_size(ctx->dtype);
  const int64_t bytes = state_block_bytes(ctx);
  *alloc = nullptr;
  if (bytes > 0 && hipMalloc(alloc, static_cast<size_t>(bytes)) != hipSuccess) {
    (void)hipGetLastError();
    *alloc = nullptr;
    return GAC_ERR_ALLOC;
  }
  ptrs->assign(ctx->n_tensors, nullptr);
  int64_t off = 0;
  for (int j = 0; j < ctx->n_tensors; ++j) {
    (*ptrs)[j] = static_cast<char*>(*alloc) + off;
    off += (ctx->numel[j] * es + 255) / 256 * 256;
  }
  return GAC_OK;
}

StepEvents* next_events(gac_ctx* ctx) {
  if (!ctx->profiling || ctx->prof_used >= static_cast<size_t>(kMaxProfiledSteps)) return nullptr;
  if (ctx->prof_used == ctx->prof_pool.size()) {
    StepEvents ev;
    for (auto& e : ev.e)
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
    ctx->prof_pool.push_back(ev);
  }
  return &ctx->prof_pool[ctx->prof_used++];
}

// The finalize step (the tail of pass 1) writes the result record into pinned host memory itself; an event
// recorded right after it lets the host learn the regime while the apply kernel still runs.
int mark_result(gac_ctx* ctx, hipStream_t stream) {
  GAC_HIP(ctx, hipEventRecord(ctx->result_event, stream));
  return GAC_OK;
}

int wait_result(gac_ctx* ctx, gac_result* host_out) {
  GAC_HIP(ctx, hipEventSynchronize(ctx->result_event));
  *host_out = *ctx->pinned_result;
  return host_out->nonfinite ? GAC_ERR_NONFINITE : GAC_OK;
}

// Reads the device-side step counter (waits for the stream's work first).
int read_step(gac_ctx* ctx, hipStream_t stream, int64_t* out) {
  GAC_HIP(ctx, hipStreamSynchronize(stream));
  GAC_HIP(ctx, hipMemcpy(out, ctx->dev_step, sizeof(int64_t), hipMemcpyDeviceToHost));
  return GAC_OK;
}

DecideParams decide_params(const gac_ctx* ctx) {
  DecideParams p;
  p.c_low = ctx->c_low;
  p.c_high = ctx->c_high;
  p.eps = ctx->eps;
  p.beta = ctx->beta;
  p.max_grad_norm = ctx->max_grad_norm;
  p.step = ctx->dev_step;
  p.hist_c = ctx->hist_c;
  p.hist_regime = ctx->hist_regime;
  p.hist_cap = ctx->hist_cap;
  p.step_value = 0;
  p.cur = ctx->snapshot ? ctx->dev_cur : nullptr;
  p.work = ctx->dev_work;
  return p;
}

int state_op(gac_ctx* ctx, int op, const void* const* src, void* const* dst, hipStream_t stream) {
  int rc = upload_state_segs(ctx, src, dst, stream);
  if (rc != GAC_OK) return rc;
  GAC_HIP(ctx, gac::launch_state_op(ctx->dtype, op, ctx->dev_segs_state, ctx->n_chunks, ctx->chunk_elems,
                                    ctx->grid_state, stream));
  return GAC_OK;
}

// Pass 1 of whichever form the context has.
int launch_pass1(gac_ctx* ctx, double* sums_out, gac_result* host_res, int mode, hipStream_t stream) {
  if (ctx->snapshot) {
    GAC_HIP(ctx, gac::launch_snap_reduce(ctx->dtype, ctx->dev_segs, ctx->n_chunks, ctx->chunk_elems,
                                         ctx->snap_buf, ctx->grid_snap, sums_out, ctx->dev_result,
                                         host_res, decide_params(ctx), mode, ctx->snap_delta, stream));
  } else {
    GAC_HIP(ctx, gac::launch_reduce(ctx->dtype, ctx->dev_segs, ctx->n_chunks, ctx->chunk_elems,
                                    ctx->dev_partials, ctx->dev_ticket, ctx->grid, sums_out,
                                    ctx->dev_result, host_res, decide_params(ctx), mode, stream));
  }
  return GAC_OK;
}

// Steps shared by gac_step / gac_apply / gac_step_adamw / gac_step_exchange.
enum class ApplyKind { kPlain, kAdamW, kExchange };

int run_step(gac_ctx* ctx, void* const* grad_ptrs, bool do_reduce, const double* sums_in,
             ApplyKind kind, const AdamScalars* adam, hipStream_t stream, gac_result* host_out) {
  int rc = upload_segs(ctx, const_cast<const void* const*>(grad_ptrs), ctx->state.data(), stream);
  if (rc != GAC_OK) return rc;
  StepEvents* ev = next_events(ctx);
  if (ev) GAC_HIP(ctx, hipEventRecord(ev->e[0], stream));
  gac_result* host_res = host_out ? ctx->pinned_result_dev : nullptr;
  if (do_reduce) {
    // the last workgroup of the reduction to finish also decides the regime
    rc = launch_pass1(ctx, ctx->dev_sums, host_res, /*mode=*/2, stream);
    if (rc != GAC_OK) return rc;
    if (ev) GAC_HIP(ctx, hipEventRecord(ev->e[1], stream));
  } else {
    if (ev) GAC_HIP(ctx, hipEventRecord(ev->e[1], stream));
    GAC_HIP(ctx, gac::launch_finalize(sums_in, ctx->dev_sums, ctx->dev_result, host_res,
                                      decide_params(ctx), stream));
  }
  if (host_out != nullptr) {
    rc = mark_result(ctx, stream);
    if (rc != GAC_OK) return rc;
  }
  if (ev) GAC_HIP(ctx, hipEventRecord(ev->e[2], stream));
  if (kind == ApplyKind::kExchange) {
    GAC_HIP(ctx, gac::launch_exchange(ctx->dtype, ctx->dev_segs, ctx->n_tensors, ctx->n_chunks,
                                      ctx->chunk_elems, ctx->dev_result, ctx->dev_work, ctx->grid_apply,
                                      stream));
  } else if (kind == ApplyKind::kPlain && ctx->snapshot) {
    GAC_HIP(ctx, gac::launch_snap_apply(ctx->dtype, ctx->dev_segs, ctx->n_tensors, ctx->n_chunks,
                                        ctx->chunk_elems, ctx->dev_result, ctx->dev_work, ctx->dev_cur,
                                        ctx->snap_delta, ctx->grid_apply, stream));
  } else if (kind == ApplyKind::kPlain) {
    GAC_HIP(ctx, gac::launch_apply(ctx->dtype, ctx->dev_segs, ctx->n_tensors, ctx->n_chunks,
                                   ctx->chunk_elems, ctx->dev_result, ctx->dev_work, ctx->grid_apply,
                                   stream));
  } else {
    GAC_HIP(ctx, gac::launch_apply_adamw(ctx->dtype, ctx->dev_segs, ctx->dev_adam, ctx->n_tensors,
                                         ctx->n_chunks, ctx->chunk_elems, ctx->dev_result,
                                         ctx->dev_work, *adam, ctx->grid_adamw, stream));
  }
  if (ev) GAC_HIP(ctx, hipEventRecord(ev->e[3], stream));
  if (host_out != nullptr) return wait_result(ctx, host_out);
  return GAC_OK;
}

// Which of the two state buffers of the snapshot form is current (waits for the stream).
int read_cur(gac_ctx* ctx, hipStream_t stream, int32_t* out) {
  *out = 0;
  if (!ctx->snapshot) return GAC_OK;
  GAC_HIP(ctx, hipStreamSynchronize(stream));
  GAC_HIP(ctx, hipMemcpy(out, ctx->dev_cur, sizeof(int32_t), hipMemcpyDeviceToHost));
  return GAC_OK;
}

}  // namespace

extern "C" {

void gac_default_config(gac_config* cfg) {
  if (cfg == nullptr) return;
  std::memset(cfg, 0, sizeof(*cfg));
  cfg->c_low = 0.05;
  cfg->c_high = 0.3;
  cfg->eps = 1e-8;
  cfg->beta = 1.0;
  cfg->dtype = GAC_BF16;
  cfg->device = -1;
}

int gac_plan_query(const int64_t* numel, int32_t n_tensors, int32_t dtype, int32_t chunk_elems,
                   int64_t* n_chunks_out, int64_t* total_numel_out) {
  if (n_tensors < 0 || (n_tensors > 0 && numel == nullptr)) return GAC_ERR_INVALID_ARG;
  int ce = 0;
  int rc = resolve_chunk_elems(dtype, chunk_elems, &ce);
  if (rc != GAC_OK) return rc;
  std::vector<int64_t> fc;
  int64_t total = 0;
  rc = plan(numel, n_tensors, ce, &fc, &total);
  if (rc != GAC_OK) return rc;
  if (n_chunks_out) *n_chunks_out = fc[n_tensors];
  if (total_numel_out) *total_numel_out = total;
  return GAC_OK;
}

namespace {
int init_impl(gac_ctx** out, const gac_config* cfg);
}

int gac_init(gac_ctx** out, const gac_config* cfg) {
  if (out == nullptr) return GAC_ERR_INVALID_ARG;
  *out = nullptr;
  try {  // host containers may throw; nothing may cross the C boundary
    return init_impl(out, cfg);
  } catch (...) {
    *out = nullptr;
    return GAC_ERR_ALLOC;
  }
}

namespace {
int init_impl(gac_ctx** out, const gac_config* cfg) {
  if (cfg == nullptr || cfg->n_tensors < 0 || (cfg->n_tensors > 0 && cfg->numel == nullptr) ||
      (cfg->flags & ~GAC_FLAG_SNAPSHOT_IN_REDUCE) != 0 || cfg->grid_blocks < 0 || cfg->grid_blocks > gac::kMaxGridBlocks ||
      cfg->apply_blocks < 0 || cfg->apply_blocks > gac::kMaxGridBlocks || cfg->reserved != 0 ||
      cfg->history_capacity < 0 || cfg->history_capacity > gac::kMaxHistory)
    return GAC_ERR_INVALID_ARG;
  if (!thresholds_ok(cfg->c_low, cfg->c_high) || !(cfg->eps >= 0.0) || !(cfg->beta >= 0.0) ||
      !std::isfinite(cfg->eps) || !std::isfinite(cfg->beta) || !(cfg->max_grad_norm >= 0.0))
    return GAC_ERR_BAD_THRESHOLDS;
  int chunk_elems = 0;
  int rc = resolve_chunk_elems(cfg->dtype, cfg->chunk_elems, &chunk_elems);
  if (rc != GAC_OK) return rc;

  gac_ctx* ctx = new (std::nothrow) gac_ctx();
  if (ctx == nullptr) return GAC_ERR_ALLOC;
  struct Cleanup {
    gac_ctx* c;
    ~Cleanup() { if (c) gac_destroy(c); }
  } cleanup{ctx};

  ctx->dtype = cfg->dtype;
  ctx->n_tensors = cfg->n_tensors;
  ctx->chunk_elems = chunk_elems;
  ctx->c_low = cfg->c_low;
  ctx->c_high = cfg->c_high;
  ctx->eps = cfg->eps;
  ctx->beta = cfg->beta;
  ctx->max_grad_norm = cfg->max_grad_norm;
  ctx->hist_cap = cfg->history_capacity > 0 ? cfg->history_capacity : 1024;
  const int n = cfg->n_tensors;
  ctx->numel.assign(cfg->numel, cfg->numel + n);
  rc = plan(ctx->numel.data(), n, chunk_elems, &ctx->first_chunk, &ctx->total);
  if (rc != GAC_OK) return rc;
  ctx->n_chunks = ctx->first_chunk[n];
  if (cfg->state_ptrs != nullptr) {
    for (int j = 0; j < n; ++j)
      if (ctx->numel[j] > 0 && cfg->state_ptrs[j] == nullptr) return GAC_ERR_INVALID_ARG;
  }
  ctx->snapshot = (cfg->flags & GAC_FLAG_SNAPSHOT_IN_REDUCE) != 0;
  if (ctx->snapshot && cfg->state_ptrs != nullptr) return GAC_ERR_INVALID_ARG;  // needs two buffers of its own

  // ---- from here on the GPU is touched
  int dev = cfg->device;
  if (dev < 0) GAC_HIP(ctx, hipGetDevice(&dev));
  ctx->device = dev;
  DeviceGuard guard(dev);
  {  // set-up for gac_step_static: resolve this device's copy of the static array once, here
    gac::StaticScratch sc;
    GAC_HIP(ctx, gac::static_scratch(dev, &sc));
  }
  hipDeviceProp_t prop;
  GAC_HIP(ctx, hipGetDeviceProperties(&prop, dev));
  auto pick_grid = [&](int requested, int64_t by_default) {
    int64_t g = requested > 0 ? requested : by_default;
    if (g > ctx->n_chunks) g = ctx->n_chunks;
    if (g < 1) g = 1;
    if (g > gac::kMaxGridBlocks) g = gac::kMaxGridBlocks;
    return static_cast<int>(g);
  };
  // Default grids, from measurements on MI355X: the reduction (static striding, one partial
  // sum per workgroup) does best with one workgroup per CU, the in-place pass (chunks drawn
  // from a counter) with workgroups on 7/8 of the CUs; more requesters lower the achieved
  // HBM bandwidth.
  const int64_t cus = prop.multiProcessorCount;
  ctx->cus = static_cast<int>(cus);
  ctx->apply_blocks_fixed = cfg->apply_blocks > 0;
  ctx->grid = pick_grid(cfg->grid_blocks, cus);
  ctx->grid_state = pick_grid(0, cus * 4);
  ctx->grid_apply = pick_grid(cfg->apply_blocks, cus * 7 / 8);
  ctx->grid_adamw = pick_grid(cfg->apply_blocks, cus * gac::adamw_blocks_per_cu(ctx->dtype));

  ctx->state.assign(n, nullptr);
  if (cfg->state_ptrs != nullptr) {
    for (int j = 0; j < n; ++j) ctx->state[j] = cfg->state_ptrs[j];
    ctx->state_is_callers = true;
  } else {
    rc = alloc_state_block(ctx, &ctx->state_alloc, &ctx->state);
    if (rc != GAC_OK) return rc;
    if (ctx->snapshot) {
      rc = alloc_state_block(ctx, &ctx->state1_alloc, &ctx->state1);
      if (rc != GAC_OK) return rc;
      ctx->snap_delta = static_cast<char*>(ctx->state1_alloc) - static_cast<char*>(ctx->state_alloc);
    }
  }
  rc = check_ptrs(ctx, const_cast<const void* const*>(ctx->state.data()));
  if (rc != GAC_OK) return rc;

  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_segs), sizeof(Seg) * (n + 1)));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_segs_state), sizeof(Seg) * (n + 1)));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_adam), sizeof(AdamSeg) * (n > 0 ? n : 1)));
  for (int s = 0; s < kPinnedSlots; ++s) {
    GAC_HIP(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned_segs[s]), sizeof(Seg) * (n + 1), hipHostMallocDefault));
    GAC_HIP(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned_adam[s]), sizeof(AdamSeg) * (n > 0 ? n : 1), hipHostMallocDefault));
    GAC_HIP(ctx, hipEventCreateWithFlags(&ctx->slot_event[s], hipEventDisableTiming));
  }
  ctx->cached_a.assign(n, nullptr);
  ctx->cached_b.assign(n, nullptr);
  ctx->cached_adam.assign(n, AdamSeg{nullptr, nullptr, nullptr, nullptr});
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_partials), sizeof(double) * 3 * ctx->grid));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_ticket), sizeof(unsigned int)));
  GAC_HIP(ctx, gac::launch_set_word(ctx->dev_ticket, 0u, nullptr));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_work), sizeof(unsigned long long)));
  GAC_HIP(ctx, gac::launch_set_step(reinterpret_cast<int64_t*>(ctx->dev_work), 0, nullptr));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_cur), sizeof(int32_t)));
  GAC_HIP(ctx, gac::launch_set_word(reinterpret_cast<uint32_t*>(ctx->dev_cur), 0u, nullptr));
  if (ctx->snapshot) {
    // working memory of the snapshot form's pass 1, in one allocation:
    // [chunk sums | group sums | ticket word | chunk counter]
    const int64_t n_groups = gac::snap_group_count(ctx->n_chunks);
    const size_t chunk_bytes = sizeof(double) * 3 * static_cast<size_t>(ctx->n_chunks > 0 ? ctx->n_chunks : 1);
    const size_t group_bytes = sizeof(double) * 3 * static_cast<size_t>(n_groups > 0 ? n_groups : 1);
    const size_t total = chunk_bytes + group_bytes + 16;
    GAC_HIP(ctx, hipMalloc(&ctx->snap_alloc, total));
    GAC_HIP(ctx, hipMemset(ctx->snap_alloc, 0, total));  // set-up: the counters start at zero
    char* base = static_cast<char*>(ctx->snap_alloc);
    ctx->snap_buf.chunk_sums = reinterpret_cast<double*>(base);
    ctx->snap_buf.group_sums = reinterpret_cast<double*>(base + chunk_bytes);
    ctx->snap_buf.ticket = reinterpret_cast<unsigned int*>(base + chunk_bytes + group_bytes);
    ctx->snap_buf.draw = reinterpret_cast<unsigned long long*>(base + chunk_bytes + group_bytes + 8);
    ctx->grid_snap = pick_grid(cfg->grid_blocks, cus);
  }
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_sums), sizeof(double) * 3));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_result), sizeof(gac_result)));
  GAC_HIP(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned_result), sizeof(gac_result),
                             hipHostMallocMapped));
  GAC_HIP(ctx, hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->pinned_result_dev),
                                       ctx->pinned_result, 0));
  GAC_HIP(ctx, hipEventCreateWithFlags(&ctx->result_event, hipEventDisableTiming));
  std::memset(ctx->pinned_result, 0, sizeof(gac_result));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_step), sizeof(int64_t)));
  GAC_HIP(ctx, gac::launch_set_step(ctx->dev_step, 0, nullptr));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->hist_c), sizeof(double) * ctx->hist_cap));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->hist_regime), sizeof(int32_t) * ctx->hist_cap));
  GAC_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->dev_diag), sizeof(gac_diag)));
  GAC_HIP(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned_diag), sizeof(gac_diag), hipHostMallocMapped));
  GAC_HIP(ctx, hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->pinned_diag_dev), ctx->pinned_diag, 0));
  GAC_HIP(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned_sweep),
                             sizeof(int32_t) * 3 * GAC_MAX_SWEEP_PAIRS, hipHostMallocMapped));
  GAC_HIP(ctx, hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->pinned_sweep_dev), ctx->pinned_sweep, 0));

  // Algorithm 1: the reference state starts at zero.
  rc = state_op(ctx, gac::kStateZero, nullptr, ctx->state.data(), nullptr);
  if (rc != GAC_OK) return rc;
  if (ctx->snapshot) {  // the spare buffer is written before it is read; zeroed for tidiness
    rc = state_op(ctx, gac::kStateZero, nullptr, ctx->state1.data(), nullptr);
    if (rc != GAC_OK) return rc;
  }
  GAC_HIP(ctx, hipStreamSynchronize(nullptr));

  cleanup.c = nullptr;
  *out = ctx;
  return GAC_OK;
}
}  // namespace

void gac_destroy(gac_ctx* ctx) {
  if (ctx == nullptr) return;
  {
    DeviceGuard guard(ctx->device);
    (void)hipDeviceSynchronize();
    if (ctx->state_alloc) (void)hipFree(ctx->state_alloc);
    if (ctx->state1_alloc) (void)hipFree(ctx->state1_alloc);
    if (ctx->snap_alloc) (void)hipFree(ctx->snap_alloc);
    if (ctx->dev_ticket) (void)hipFree(ctx->dev_ticket);
    if (ctx->dev_cur) (void)hipFree(ctx->dev_cur);
    if (ctx->dev_work) (void)hipFree(ctx->dev_work);
    if (ctx->dev_segs) (void)hipFree(ctx->dev_segs);
    if (ctx->dev_segs_state) (void)hipFree(ctx->dev_segs_state);
    if (ctx->dev_adam) (void)hipFree(ctx->dev_adam);
    if (ctx->dev_partials) (void)hipFree(ctx->dev_partials);
    if (ctx->dev_sums) (void)hipFree(ctx->dev_sums);
    if (ctx->dev_result) (void)hipFree(ctx->dev_result);
    if (ctx->pinned_result) (void)hipHostFree(ctx->pinned_result);
    if (ctx->dev_step) (void)hipFree(ctx->dev_step);
    if (ctx->hist_c) (void)hipFree(ctx->hist_c);
    if (ctx->hist_regime) (void)hipFree(ctx->hist_regime);
    if (ctx->dev_diag) (void)hipFree(ctx->dev_diag);
    if (ctx->pinned_diag) (void)hipHostFree(ctx->pinned_diag);
    if (ctx->pinned_sweep) (void)hipHostFree(ctx->pinned_sweep);
    if (ctx->result_event) (void)hipEventDestroy(ctx->result_event);
    for (int s = 0; s < kPinnedSlots; ++s) {
      if (ctx->pinned_segs[s]) (void)hipHostFree(ctx->pinned_segs[s]);
      if (ctx->pinned_adam[s]) (void)hipHostFree(ctx->pinned_adam[s]);
      if (ctx->slot_event[s]) (void)hipEventDestroy(ctx->slot_event[s]);
    }
    for (auto& ev : ctx->prof_pool)
      for (auto& e : ev.e) (void)hipEventDestroy(e);
  }
  delete ctx;
}

int gac_step(gac_ctx* ctx, void* const* grad_ptrs, void* hip_stream, gac_result* host_out) {
  if (ctx == nullptr) return GAC_ERR_INVALID_ARG;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(grad_ptrs));
  if (rc == GAC_OK) rc = check_not_state(ctx, grad_ptrs);
  if (rc != GAC_OK) return rc;
  DeviceGuard guard(ctx->device);
  return run_step(ctx, grad_ptrs, true, nullptr, ApplyKind::kPlain, nullptr,
                  static_cast<hipStream_t>(hip_stream), host_out);
}

int gac_step_exchange(gac_ctx* ctx, void** grad_ptrs, void* hip_stream, gac_result* host_out) {
  if (ctx == nullptr || host_out == nullptr || !ctx->state_is_callers) return GAC_ERR_INVALID_ARG;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(grad_ptrs));
  if (rc == GAC_OK) rc = check_not_state(ctx, grad_ptrs);
  if (rc != GAC_OK) return rc;
  DeviceGuard guard(ctx->device);
  rc = run_step(ctx, grad_ptrs, true, nullptr, ApplyKind::kExchange, nullptr,
                static_cast<hipStream_t>(hip_stream), host_out);
  if (rc != GAC_OK) return rc;  // includes the non-finite case: no buffer changes hands
  for (int j = 0; j < ctx->n_tensors; ++j) {
    void* old_state = ctx->state[j];
    ctx->state[j] = grad_ptrs[j];
    grad_ptrs[j] = old_state;
  }
  return GAC_OK;
}

int gac_reduce_local(gac_ctx* ctx, void* const* grad_ptrs, void* hip_stream, double* dev_sums3) {
  if (ctx == nullptr || dev_sums3 == nullptr) return GAC_ERR_INVALID_ARG;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(grad_ptrs));
  if (rc != GAC_OK) return rc;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  rc = upload_segs(ctx, const_cast<const void* const*>(grad_ptrs), ctx->state.data(), stream);
  if (rc != GAC_OK) return rc;
  // sums only: the regime is decided in phase 2, on the global sums
  rc = launch_pass1(ctx, dev_sums3, nullptr, /*mode=*/0, stream);
  if (rc != GAC_OK) return rc;
  return GAC_OK;
}

int gac_apply(gac_ctx* ctx, void* const* grad_ptrs, const double* dev_sums3, void* hip_stream,
              gac_result* host_out) {
  if (ctx == nullptr || dev_sums3 == nullptr) return GAC_ERR_INVALID_ARG;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(grad_ptrs));
  if (rc == GAC_OK) rc = check_not_state(ctx, grad_ptrs);
  if (rc != GAC_OK) return rc;
  DeviceGuard guard(ctx->device);
  return run_step(ctx, grad_ptrs, false, dev_sums3, ApplyKind::kPlain, nullptr,
                  static_cast<hipStream_t>(hip_stream), host_out);
}

int gac_step_adamw(gac_ctx* ctx, void* const* grad_ptrs, float* const* master_p, float* const* m,
                   float* const* v, void* const* p_lowp, const gac_adamw_hyper* hyper,
                   void* hip_stream, gac_result* host_out) {
  if (ctx == nullptr || hyper == nullptr) return GAC_ERR_INVALID_ARG;
  if (ctx->snapshot) return GAC_ERR_UNIMPLEMENTED;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(grad_ptrs));
  if (rc == GAC_OK) rc = check_not_state(ctx, grad_ptrs);
  if (rc != GAC_OK) return rc;
  if (ctx->n_tensors > 0 && (master_p == nullptr || m == nullptr || v == nullptr)) return GAC_ERR_INVALID_ARG;
  for (int j = 0; j < ctx->n_tensors; ++j) {
    if (ctx->numel[j] == 0) continue;
    if (!master_p[j] || !m[j] || !v[j]) return GAC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(master_p[j]) | reinterpret_cast<uintptr_t>(m[j]) |
         reinterpret_cast<uintptr_t>(v[j])) & 3u)
      return GAC_ERR_INVALID_ARG;
    if (p_lowp != nullptr && (p_lowp[j] == nullptr || reinterpret_cast<uintptr_t>(p_lowp[j]) %
                                                          static_cast<uintptr_t>(elem_size(ctx->dtype))))
      return GAC_ERR_INVALID_ARG;
  }
  if (hyper->t_adam < 1 || !(hyper->beta1 >= 0 && hyper->beta1 < 1) ||
      !(hyper->beta2 >= 0 && hyper->beta2 < 1) || !(hyper->eps_adam >= 0) ||
      !std::isfinite(hyper->lr) || !std::isfinite(hyper->weight_decay))
    return GAC_ERR_INVALID_ARG;
  AdamScalars h;
  const double bc1 = 1.0 - std::pow(hyper->beta1, static_cast<double>(hyper->t_adam));
  const double bc2 = 1.0 - std::pow(hyper->beta2, static_cast<double>(hyper->t_adam));
  h.beta1 = static_cast<float>(hyper->beta1);
  h.one_minus_beta1 = static_cast<float>(1.0 - hyper->beta1);
  h.beta2 = static_cast<float>(hyper->beta2);
  h.one_minus_beta2 = static_cast<float>(1.0 - hyper->beta2);
  h.lr_wd = static_cast<float>(hyper->lr * hyper->weight_decay);
  h.step_size = static_cast<float>(hyper->lr / bc1);
  h.inv_sqrt_bc2 = static_cast<float>(1.0 / std::sqrt(bc2));
  h.eps_adam = static_cast<float>(hyper->eps_adam);
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  rc = upload_adam(ctx, master_p, m, v, p_lowp, stream);
  if (rc != GAC_OK) return rc;
  return run_step(ctx, grad_ptrs, true, nullptr, ApplyKind::kAdamW, &h, stream, host_out);
}

int gac_result_device(const gac_ctx* ctx, const gac_result** dev_ptr) {
  if (ctx == nullptr || dev_ptr == nullptr) return GAC_ERR_INVALID_ARG;
  *dev_ptr = ctx->dev_result;
  return GAC_OK;
}

int gac_state_export(gac_ctx* ctx, void* const* dst_ptrs, int64_t* step_out, void* hip_stream) {
  if (ctx == nullptr) return GAC_ERR_INVALID_ARG;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(dst_ptrs));
  if (rc != GAC_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (step_out) {
    rc = read_step(ctx, static_cast<hipStream_t>(hip_stream), step_out);
    if (rc != GAC_OK) return rc;
  }
  int32_t cur = 0;
  rc = read_cur(ctx, static_cast<hipStream_t>(hip_stream), &cur);
  if (rc != GAC_OK) return rc;
  const std::vector<void*>& src = cur ? ctx->state1 : ctx->state;
  return state_op(ctx, gac::kStateCopy, const_cast<const void* const*>(src.data()), dst_ptrs,
                  static_cast<hipStream_t>(hip_stream));
}

int gac_state_import(gac_ctx* ctx, void* const* src_ptrs, int64_t step, void* hip_stream) {
  if (ctx == nullptr || step < 0) return GAC_ERR_INVALID_ARG;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(src_ptrs));
  if (rc != GAC_OK) return rc;
  DeviceGuard guard(ctx->device);
  rc = state_op(ctx, gac::kStateCopy, const_cast<const void* const*>(src_ptrs), ctx->state.data(),
                static_cast<hipStream_t>(hip_stream));
  if (rc == GAC_OK) {
    GAC_HIP(ctx, gac::launch_set_step(ctx->dev_step, step, static_cast<hipStream_t>(hip_stream)));
    // snapshot form: the imported state went into buffer 0, which becomes the current one
    GAC_HIP(ctx, gac::launch_set_word(reinterpret_cast<uint32_t*>(ctx->dev_cur), 0u,
                                      static_cast<hipStream_t>(hip_stream)));
    ctx->hist_first = step + 1;
  }
  return rc;
}

int gac_reset(gac_ctx* ctx, void* hip_stream) {
  if (ctx == nullptr) return GAC_ERR_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  int rc = state_op(ctx, gac::kStateZero, nullptr, ctx->state.data(), static_cast<hipStream_t>(hip_stream));
  if (rc == GAC_OK) {
    GAC_HIP(ctx, gac::launch_set_step(ctx->dev_step, 0, static_cast<hipStream_t>(hip_stream)));
    GAC_HIP(ctx, gac::launch_set_word(reinterpret_cast<uint32_t*>(ctx->dev_cur), 0u,
                                      static_cast<hipStream_t>(hip_stream)));
    ctx->hist_first = 1;
  }
  return rc;
}

namespace {
// Median time of three launches (after one untimed) of the in-place probe, or of the
// reduction pass when `reduce` is set, with the state at `state_ptrs`.
int time_probe(gac_ctx* ctx, void* const* grad_ptrs, void* const* state_ptrs, bool reduce, int grid,
               hipStream_t stream, hipEvent_t e0, hipEvent_t e1, double* ms_out) {
  int rc = upload_segs(ctx, const_cast<const void* const*>(grad_ptrs), state_ptrs, stream);
  if (rc != GAC_OK) return rc;
  float ms[3];
  for (int i = -1; i < 3; ++i) {
    GAC_HIP(ctx, hipEventRecord(e0, stream));
    if (reduce) {
      // sums only (mode 0): no step is counted and no result is written
      GAC_HIP(ctx, gac::launch_reduce(ctx->dtype, ctx->dev_segs, ctx->n_chunks, ctx->chunk_elems,
                                      ctx->dev_partials, ctx->dev_ticket, ctx->grid, ctx->dev_sums,
                                      ctx->dev_result, nullptr, decide_params(ctx), /*mode=*/0,
                                      stream));
    } else {
      GAC_HIP(ctx, gac::launch_set_step(reinterpret_cast<int64_t*>(ctx->dev_work), 0, stream));
      GAC_HIP(ctx, gac::launch_apply_probe(ctx->dtype, ctx->dev_segs, ctx->n_tensors, ctx->n_chunks,
                                           ctx->chunk_elems, ctx->dev_work, grid, stream));
    }
    GAC_HIP(ctx, hipEventRecord(e1, stream));
    GAC_HIP(ctx, hipEventSynchronize(e1));
    if (i >= 0) GAC_HIP(ctx, hipEventElapsedTime(&ms[i], e0, e1));
  }
  const float lo = ms[0] < ms[1] ? ms[0] : ms[1], hi = ms[0] < ms[1] ? ms[1] : ms[0];
  *ms_out = ms[2] < lo ? lo : (ms[2] > hi ? hi : ms[2]);
  return GAC_OK;
}

// Both passes of a step with the state at one candidate location.
int time_candidate(gac_ctx* ctx, void* const* grad_ptrs, void* const* state_ptrs, hipStream_t stream,
                   hipEvent_t e0, hipEvent_t e1, double* probe_ms, double* reduce_ms) {
  int rc = time_probe(ctx, grad_ptrs, state_ptrs, false, ctx->grid_apply, stream, e0, e1, probe_ms);
  if (rc == GAC_OK) rc = time_probe(ctx, grad_ptrs, state_ptrs, true, 0, stream, e0, e1, reduce_ms);
  return rc;
}

struct Candidate {
  void* alloc = nullptr;
  std::vector<void*> ptrs;
};

int place_state_impl(gac_ctx* ctx, void* const* grad_ptrs, int32_t max_candidates,
                     int64_t max_extra_bytes, hipStream_t stream, gac_placement* rep) {
  constexpr int64_t kMinBytes = 256ll << 20, kReserve = 4ll << 30;
  // Successive candidates start at least this much deeper in memory than the one before
  // (the regions that matter are ~90 GiB wide); a state smaller than the stride gets spacers,
  // allocated in pieces small enough for the driver to pack them one after the other.
  constexpr int64_t kStride = 12ll << 30, kSpacerPiece = 1ll << 30;
  rep->n_candidates = 1;
  rep->chosen = 0;
  rep->apply_blocks = ctx->grid_apply;
  const int64_t bytes = state_block_bytes(ctx);
  if (bytes < kMinBytes) return GAC_OK;
  GAC_HIP(ctx, hipStreamSynchronize(stream));
  // Everything the search holds; whatever is still here when it goes out of scope (also on
  // an error or an exception) is released, except the candidate that became the state.
  struct Search {
    std::vector<Candidate> cand;
    std::vector<void*> spacers;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int keep = -1;
    ~Search() {
      for (int c = 1; c < static_cast<int>(cand.size()); ++c)
        if (c != keep && cand[c].alloc) (void)hipFree(cand[c].alloc);
      for (void* sp : spacers) (void)hipFree(sp);
      if (e0) (void)hipEventDestroy(e0);
      if (e1) (void)hipEventDestroy(e1);
    }
  } search;
  GAC_HIP(ctx, hipEventCreate(&search.e0));
  GAC_HIP(ctx, hipEventCreate(&search.e1));
  std::vector<Candidate>& cand = search.cand;
  std::vector<void*>& spacers = search.spacers;
  const hipEvent_t e0 = search.e0, e1 = search.e1;
  cand.reserve(GAC_MAX_PLACEMENT_CANDIDATES);  // no reallocation between an allocation and its record
  spacers.reserve(static_cast<size_t>(GAC_MAX_PLACEMENT_CANDIDATES * (kStride / kSpacerPiece)));
  cand.resize(1);
  cand[0].alloc = ctx->state_alloc;
  cand[0].ptrs = ctx->state;
  // On any failure the pointer table goes back to (grad_ptrs, current state): a graph captured
  // earlier must never replay against a candidate that has been freed.
  auto fail = [&](int code) {
    ctx->segs_valid = false;
    (void)upload_segs(ctx, const_cast<const void* const*>(grad_ptrs), ctx->state.data(), stream);
    (void)hipStreamSynchronize(stream);
    return code;
  };
  int rc = time_candidate(ctx, grad_ptrs, cand[0].ptrs.data(), stream, e0, e1, &rep->probe_ms[0],
                          &rep->reduce_ms[0]);
  int64_t extra = 0;
  // The search ends early once a clearly better location (3 %) has been followed by two
  // that are no better, or after eight in a row without any gain: every candidate is memory
  // the driver has to take back afterwards.
  double best_sum = rep->probe_ms[0] + rep->reduce_ms[0];
  const double first_sum = best_sum;
  int since_best = 0;
  while (rc == GAC_OK && static_cast<int>(cand.size()) < max_candidates) {
    if (since_best >= 2 && best_sum < 0.97 * first_sum) break;
    if (since_best >= 8) break;  // a whole region (8 strides) without any gain: nothing to find
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) {
      (void)hipGetLastError();
      break;
    }
    const int64_t gap = bytes < kStride ? kStride - bytes : 0;
    if (static_cast<int64_t>(free_b) < gap + bytes + kReserve) break;
    if (max_extra_bytes > 0 && extra + gap + bytes > max_extra_bytes) break;
    bool spaced = true;
    for (int64_t done = 0; done < gap && spaced; done += kSpacerPiece) {
      void* sp = nullptr;
      const int64_t piece = gap - done < kSpacerPiece ? gap - done : kSpacerPiece;
      if (hipMalloc(&sp, static_cast<size_t>(piece)) != hipSuccess) {
        (void)hipGetLastError();
        spaced = false;
      } else {
        spacers.push_back(sp);
        extra += piece;
      }
    }
    if (!spaced) break;
    Candidate c;
    if (alloc_state_block(ctx, &c.alloc, &c.ptrs) != GAC_OK) break;  // out of memory: stop quietly
    extra += bytes;
    cand.push_back(c);
    const int i = static_cast<int>(cand.size()) - 1;
    rc = time_candidate(ctx, grad_ptrs, cand[i].ptrs.data(), stream, e0, e1, &rep->probe_ms[i],
                        &rep->reduce_ms[i]);
    const double sum = rep->probe_ms[i] + rep->reduce_ms[i];
    if (sum < 0.995 * best_sum) {
      best_sum = sum;
      since_best = 0;
    } else {
      ++since_best;
    }
  }
  rep->bytes_held_peak = extra;  // nothing is released before the end of the search
  if (rc != GAC_OK) return fail(rc);
  rep->n_candidates = static_cast<int>(cand.size());
  auto both = [&](int c) { return rep->probe_ms[c] + rep->reduce_ms[c]; };
  int best = 0;
  for (int c = 1; c < rep->n_candidates; ++c)
    if (both(c) < both(best)) best = c;
  if (both(best) > 0.99 * both(0)) best = 0;  // not worth a move
  if (best != 0) {
    rc = state_op(ctx, gac::kStateCopy, const_cast<const void* const*>(ctx->state.data()),
                  cand[best].ptrs.data(), stream);
    if (rc == GAC_OK && hipStreamSynchronize(stream) != hipSuccess) rc = fail_hip(ctx, hipGetLastError(), "hipStreamSynchronize");
    if (rc != GAC_OK) return fail(rc);
    (void)hipFree(ctx->state_alloc);
    search.keep = best;
    ctx->state_alloc = cand[best].alloc;
    ctx->state = cand[best].ptrs;
  }
  rep->chosen = best;
  // workgroup count of the in-place pass at the chosen location
  if (!ctx->apply_blocks_fixed) {
    const int64_t tries[4] = {ctx->cus * 3ll / 4, ctx->cus * 13ll / 16, ctx->cus * 7ll / 8, ctx->cus};
    int n = 0, best_blocks = ctx->grid_apply;
    double best_ms = 0.0;
    for (int64_t b : tries) {
      if (b < 1) b = 1;
      if (b > ctx->n_chunks) b = ctx->n_chunks;
      if (b > gac::kMaxGridBlocks) b = gac::kMaxGridBlocks;
      bool seen = false;
      for (int i = 0; i < n; ++i) seen = seen || rep->blocks_tried[i] == b;
      if (seen) continue;
      double ms = 0.0;
      rc = time_probe(ctx, grad_ptrs, ctx->state.data(), false, static_cast<int>(b), stream, e0, e1, &ms);
      if (rc != GAC_OK) break;
      rep->blocks_tried[n] = static_cast<int32_t>(b);
      rep->blocks_ms[n] = ms;
      if (n == 0 || ms < best_ms) {
        best_ms = ms;
        best_blocks = static_cast<int>(b);
      }
      ++n;
    }
    rep->n_blocks_tried = n;
    if (rc == GAC_OK) ctx->grid_apply = best_blocks;
  }
  rep->apply_blocks = ctx->grid_apply;
  if (rc != GAC_OK) return fail(rc);
  // Leave the device pointer table on (grad_ptrs, final state): a graph captured earlier reads
  // the table when it is replayed and must never see a candidate that is about to be freed.
  ctx->segs_valid = false;
  rc = upload_segs(ctx, const_cast<const void* const*>(grad_ptrs), ctx->state.data(), stream);
  if (rc == GAC_OK && hipStreamSynchronize(stream) != hipSuccess)
    rc = fail_hip(ctx, hipGetLastError(), "hipStreamSynchronize");
  return rc;
}
}  // namespace

int gac_place_state(gac_ctx* ctx, void* const* grad_ptrs, int32_t max_candidates,
                    int64_t max_extra_bytes, void* hip_stream, gac_placement* report) {
  if (ctx == nullptr || max_candidates < 1 || max_candidates > GAC_MAX_PLACEMENT_CANDIDATES ||
      max_extra_bytes < 0 || (ctx->state_is_callers && max_candidates != 1))
    return GAC_ERR_INVALID_ARG;
  if (ctx->snapshot) return GAC_ERR_UNIMPLEMENTED;
  int rc = check_ptrs(ctx, const_cast<const void* const*>(grad_ptrs));
  if (rc == GAC_OK) rc = check_not_state(ctx, grad_ptrs);
  if (rc != GAC_OK) return rc;
  DeviceGuard guard(ctx->device);
  gac_placement local;
  std::memset(&local, 0, sizeof(local));
  try {
    rc = place_state_impl(ctx, grad_ptrs, max_candidates, max_extra_bytes,
                          static_cast<hipStream_t>(hip_stream), &local);
  } catch (...) {
    rc = GAC_ERR_ALLOC;
  }
  if (report != nullptr) *report = local;
  return rc;
}

int gac_set_thresholds(gac_ctx* ctx, double c_low, double c_high) {
  if (ctx == nullptr) return GAC_ERR_INVALID_ARG;
  if (!thresholds_ok(c_low, c_high)) return GAC_ERR_BAD_THRESHOLDS;
  ctx->c_low = c_low;
  ctx->c_high = c_high;
  return GAC_OK;
}

namespace {
// Range of step numbers whose record is still in the ring.
int recorded_range(gac_ctx* ctx, hipStream_t stream, int64_t* first, int64_t* last) {
  int64_t step = 0;
  int rc = read_step(ctx, stream, &step);
  if (rc != GAC_OK) return rc;
  *last = step;
  int64_t f = step - ctx->hist_cap + 1;
  if (f < ctx->hist_first) f = ctx->hist_first;
  *first = f;
  return GAC_OK;
}
}  // namespace

int gac_history_read(gac_ctx* ctx, int64_t max_n, double* c_out, int32_t* regime_out,
                     int64_t* n_out, int64_t* first_step_out, void* hip_stream) {
  if (ctx == nullptr || max_n < 0 || n_out == nullptr) return GAC_ERR_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int64_t first, last;
  int rc = recorded_range(ctx, stream, &first, &last);
  if (rc != GAC_OK) return rc;
  int64_t n = last >= first ? last - first + 1 : 0;
  if (n > max_n) {
    first += n - max_n;
    n = max_n;
  }
  *n_out = n;
  if (first_step_out) *first_step_out = first;
  if (n == 0) return GAC_OK;
  std::vector<double> c;
  std::vector<int32_t> r;
  try {
    c.resize(ctx->hist_cap);
    r.resize(ctx->hist_cap);
  } catch (...) {
    return GAC_ERR_ALLOC;
  }
  GAC_HIP(ctx, hipMemcpy(c.data(), ctx->hist_c, sizeof(double) * ctx->hist_cap, hipMemcpyDeviceToHost));
  GAC_HIP(ctx, hipMemcpy(r.data(), ctx->hist_regime, sizeof(int32_t) * ctx->hist_cap, hipMemcpyDeviceToHost));
  for (int64_t i = 0; i < n; ++i) {
    const int slot = static_cast<int>((first + i - 1) % ctx->hist_cap);
    if (c_out) c_out[i] = c[slot];
    if (regime_out) regime_out[i] = r[slot] < 0 ? GAC_SKIP : r[slot];
  }
  return GAC_OK;
}

int gac_diag_summary(gac_ctx* ctx, int64_t burn_in, gac_diag* out, void* hip_stream) {
  if (ctx == nullptr || out == nullptr || burn_in < 0) return GAC_ERR_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int64_t first, last;
  int rc = recorded_range(ctx, stream, &first, &last);
  if (rc != GAC_OK) return rc;
  if (first < burn_in + 1) first = burn_in + 1;
  GAC_HIP(ctx, gac::launch_diag(ctx->hist_c, ctx->hist_regime, ctx->hist_cap, first, last, ctx->c_low,
                                ctx->dev_diag, ctx->pinned_diag_dev, stream));
  GAC_HIP(ctx, hipStreamSynchronize(stream));
  *out = *ctx->pinned_diag;
  return GAC_OK;
}

int gac_threshold_sweep(gac_ctx* ctx, int64_t burn_in, int32_t n_pairs, const double* c_low,
                        const double* c_high, int32_t* counts, void* hip_stream) {
  if (ctx == nullptr || c_low == nullptr || c_high == nullptr || counts == nullptr || burn_in < 0 ||
      n_pairs < 1 || n_pairs > GAC_MAX_SWEEP_PAIRS)
    return GAC_ERR_INVALID_ARG;
  gac::SweepPairs pairs;
  for (int i = 0; i < GAC_MAX_SWEEP_PAIRS; ++i) {
    const int j = i < n_pairs ? i : 0;
    if (!(c_low[j] > 0.0) || !(c_low[j] < c_high[j])) return GAC_ERR_BAD_THRESHOLDS;
    pairs.c_low[i] = c_low[j];
    pairs.c_high[i] = c_high[j];
  }
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int64_t first, last;
  int rc = recorded_range(ctx, stream, &first, &last);
  if (rc != GAC_OK) return rc;
  if (first < burn_in + 1) first = burn_in + 1;
  GAC_HIP(ctx, gac::launch_sweep(ctx->hist_c, ctx->hist_regime, ctx->hist_cap, first, last, pairs,
                                 n_pairs, ctx->pinned_sweep_dev, stream));
  GAC_HIP(ctx, hipStreamSynchronize(stream));
  std::memcpy(counts, ctx->pinned_sweep, sizeof(int32_t) * 3 * n_pairs);
  return GAC_OK;
}

int gac_profile_enable(gac_ctx* ctx, int32_t on) {
  if (ctx == nullptr) return GAC_ERR_INVALID_ARG;
  if (on) {
    try {
      ctx->prof_pool.reserve(kMaxProfiledSteps);  // so that recording a step never allocates
    } catch (...) {
      return GAC_ERR_ALLOC;
    }
  }
  ctx->profiling = on != 0;
  ctx->prof_used = 0;
  return GAC_OK;
}

int gac_profile_read(gac_ctx* ctx, double* ms_reduce, double* ms_finalize, double* ms_apply,
                     int32_t* n_steps) {
  if (ctx == nullptr) return GAC_ERR_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  double t[3] = {0, 0, 0};
  for (size_t i = 0; i < ctx->prof_used; ++i) {
    StepEvents& ev = ctx->prof_pool[i];
    GAC_HIP(ctx, hipEventSynchronize(ev.e[3]));
    for (int k = 0; k < 3; ++k) {
      float ms = 0.f;
      GAC_HIP(ctx, hipEventElapsedTime(&ms, ev.e[k], ev.e[k + 1]));
      t[k] += ms;
    }
  }
  if (ms_reduce) *ms_reduce = t[0];
  if (ms_finalize) *ms_finalize = t[1];
  if (ms_apply) *ms_apply = t[2];
  if (n_steps) *n_steps = static_cast<int32_t>(ctx->prof_used);
  ctx->prof_used = 0;
  return GAC_OK;
}

// ---- gac_step_static: the step for callers that cannot allocate (see gac.h) ----------------
namespace {
// Grid defaults are per device; looked up once (no allocation) and kept.
constexpr int kMaxDevicesStatic = 64;
int g_static_cus[kMaxDevicesStatic] = {};

int static_step_impl(const gac_config* cfg, void* const* grad_ptrs, int64_t step,
                     hipStream_t stream, gac_result* result_out) {
  if (cfg == nullptr || cfg->n_tensors < 0 || (cfg->n_tensors > 0 && (cfg->numel == nullptr ||
      cfg->state_ptrs == nullptr || grad_ptrs == nullptr)) || cfg->flags != 0 || cfg->reserved != 0 ||
      cfg->history_capacity != 0 || cfg->grid_blocks < 0 || cfg->apply_blocks < 0 ||
      cfg->apply_blocks > gac::kMaxGridBlocks || step < 0)
    return GAC_ERR_INVALID_ARG;
  if (cfg->n_tensors > gac::kStaticMaxTensors || cfg->grid_blocks > gac::kStaticMaxGrid)
    return GAC_ERR_TOO_LARGE;
  if (!thresholds_ok(cfg->c_low, cfg->c_high) || !(cfg->eps >= 0.0) || !(cfg->beta >= 0.0) ||
      !std::isfinite(cfg->eps) || !std::isfinite(cfg->beta) || !(cfg->max_grad_norm >= 0.0))
    return GAC_ERR_BAD_THRESHOLDS;
  int chunk_elems = 0;
  int rc = resolve_chunk_elems(cfg->dtype, cfg->chunk_elems, &chunk_elems);
  if (rc != GAC_OK) return rc;
  const int n = cfg->n_tensors;
  const uintptr_t es = static_cast<uintptr_t>(elem_size(cfg->dtype));
  int64_t n_chunks = 0;
  for (int j = 0; j < n; ++j) {
    if (cfg->numel[j] < 0) return GAC_ERR_INVALID_ARG;
    const uintptr_t g = reinterpret_cast<uintptr_t>(grad_ptrs[j]);
    const uintptr_t d = reinterpret_cast<uintptr_t>(cfg->state_ptrs[j]);
    if (cfg->numel[j] > 0 && (g == 0 || d == 0 || g == d)) return GAC_ERR_INVALID_ARG;
    if (g % es != 0 || d % es != 0) return GAC_ERR_INVALID_ARG;
    n_chunks += (cfg->numel[j] + chunk_elems - 1) / chunk_elems;
  }

  // ---- from here on the GPU is touched
  int dev = cfg->device;
  if (dev < 0) GAC_HIP(nullptr, hipGetDevice(&dev));
  if (dev >= kMaxDevicesStatic) return GAC_ERR_INVALID_ARG;
  DeviceGuard guard(dev);
  gac::StaticScratch sc;
  GAC_HIP(nullptr, gac::static_scratch(dev, &sc));
  if (g_static_cus[dev] == 0) {
    int cus = 0;
    GAC_HIP(nullptr, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    g_static_cus[dev] = cus > 0 ? cus : 1;
  }
  const int64_t cus = g_static_cus[dev];
  auto pick_grid = [&](int requested, int64_t by_default, int64_t cap) {
    int64_t g = requested > 0 ? requested : by_default;
    if (g > n_chunks) g = n_chunks;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return static_cast<int>(g);
  };
  // the same defaults as gac_init, so that the partial sums (and with them every bit of the
  // result) are those of gac_step
  const int grid = pick_grid(cfg->grid_blocks, cus, gac::kStaticMaxGrid);
  const int grid_apply = pick_grid(cfg->apply_blocks, cus * 7 / 8, gac::kMaxGridBlocks);

  // The tensor table goes to the device as kernel arguments, a batch at a time; the first
  // batch also clears the ticket counter (an earlier call that was cut short may have left it
  // anywhere).
  gac::SegBatch batch;
  int64_t c = 0;
  int filled = 0;
  bool first_batch = true;
  auto flush = [&](int first) -> int {
    batch.first = first;
    batch.count = filled;
    GAC_HIP(nullptr, gac::launch_fill_segs(sc.segs, batch, first_batch ? sc.ticket : nullptr, stream));
    first_batch = false;
    filled = 0;
    return GAC_OK;
  };
  int batch_first = 0;
  for (int j = 0; j <= n; ++j) {  // entry n is the sentinel
    Seg& e = batch.e[filled];
    e.a = j < n ? grad_ptrs[j] : nullptr;
    e.b = j < n ? cfg->state_ptrs[j] : nullptr;
    e.numel = j < n ? cfg->numel[j] : 0;
    e.first_chunk = c;
    if (j < n) c += (cfg->numel[j] + chunk_elems - 1) / chunk_elems;
    if (++filled == gac::kSegBatch || j == n) {
      rc = flush(batch_first);
      if (rc != GAC_OK) return rc;
      batch_first = j + 1;
    }
  }

  DecideParams p;
  p.c_low = cfg->c_low;
  p.c_high = cfg->c_high;
  p.eps = cfg->eps;
  p.beta = cfg->beta;
  p.max_grad_norm = cfg->max_grad_norm;
  p.step = nullptr;
  p.hist_c = nullptr;
  p.hist_regime = nullptr;
  p.hist_cap = 0;
  p.step_value = step;
  p.cur = nullptr;
  p.work = sc.work;
  GAC_HIP(nullptr, gac::launch_reduce(cfg->dtype, sc.segs, n_chunks, chunk_elems, sc.partials, sc.ticket,
                                      grid, sc.sums, sc.result, result_out, p, /*mode=*/2, stream));
  GAC_HIP(nullptr, gac::launch_apply(cfg->dtype, sc.segs, n, n_chunks, chunk_elems, sc.result,
                                     sc.work, grid_apply, stream));
  return GAC_OK;
}
}  // namespace

int gac_step_static(const gac_config* cfg, void* const* grad_ptrs, int64_t step, void* hip_stream,
                    gac_result* result_out) {
  return static_step_impl(cfg, grad_ptrs, step, static_cast<hipStream_t>(hip_stream), result_out);
}

const char* gac_strerror(int code) {
  switch (code) {
    case GAC_OK: return "ok";
    case GAC_ERR_INVALID_ARG: return "invalid argument";
    case GAC_ERR_BAD_THRESHOLDS: return "thresholds must satisfy 0 < c_low < c_high, eps >= 0, beta >= 0";
    case GAC_ERR_ALLOC: return "allocation failed";
    case GAC_ERR_HIP: return "HIP runtime error";
    case GAC_ERR_NONFINITE: return "non-finite gradient statistics; nothing was modified";
    case GAC_ERR_UNIMPLEMENTED: return "not implemented for this configuration";
    case GAC_ERR_TOO_LARGE: return "size exceeds a fixed capacity of the library (see gac_step_static)";
    default: return "unknown error code";
  }
}

const char* gac_last_hip_error(const gac_ctx* ctx) {
  return ctx ? ctx->hip_err.c_str() : g_last_hip_error.c_str();
}

const char* gac_version(void) { return "gac-mi355x 0.2"; }

#ifndef GAC_SOURCE_HASH
#define GAC_SOURCE_HASH ""
#endif
const char* gac_source_hash(void) { return GAC_SOURCE_HASH; }

}  // extern "C"
