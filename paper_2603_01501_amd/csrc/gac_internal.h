// Internal interface between the host side of the library (context, planner, C ABI)
// and its HIP kernels.  Not installed; the public interface is include/gac.h.
#pragma once

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "gac.h"

namespace gac {

// Default size of a chunk, in bytes of one array.  The pass-2 kernels keep whole tiles of this
// size (or a fixed fraction of it) in registers; other chunk sizes take their slower generic path.
constexpr int kDefaultChunkBytes = 65536;

// One entry per tensor plus a sentinel entry (first_chunk = total number of chunks).
// The tensor list is cut into chunks of at most chunk_elems elements; a chunk never
// straddles two tensors, so every chunk is one contiguous range of one g and one d.
struct Seg {
  const void* a;        // gradient g (reduce/apply), or source buffer (state copy)
  void* b;              // reference state d, or destination buffer (state copy)
  int64_t numel;
  int64_t first_chunk;  // index of this tensor's first chunk in the global chunk order
};
static_assert(sizeof(Seg) == 32, "Seg layout is shared with device code");

// Per-tensor optimizer buffers for the fused AdamW pass.
struct AdamSeg {
  float* p;
  float* m;
  float* v;
  void* p_lowp;  // may be null
};
static_assert(sizeof(AdamSeg) == 32, "AdamSeg layout is shared with device code");

// What the finalize step needs besides the sums.
struct DecideParams {
  double c_low, c_high, eps, beta;
  double max_grad_norm;  // 0 = no clipping
  int64_t* step;         // device-side step counter, incremented by the finalize step, so that
                         // a captured and replayed launch sequence keeps counting
  double* hist_c;        // ring of recorded cosines, hist_cap entries (or null)
  int32_t* hist_regime;  // ring of recorded regimes
  int32_t hist_cap;
  int64_t step_value;    // used when `step` is null: the number this update gets (the caller counts)
  int32_t* cur;          // snapshot form: which of the two state buffers is current (flipped by a
                         // finite step); null otherwise
  unsigned long long* work;  // the counter pass 2 draws its chunks from; the finalize step zeroes it
};

constexpr int kMaxHistory = 4096;  // the statistics kernel sorts the ring in LDS

// AdamW scalars, prepared on the host in fp64 and rounded once to fp32.
struct AdamScalars {
  float beta1, one_minus_beta1;
  float beta2, one_minus_beta2;
  float lr_wd;         // lr * weight_decay
  float step_size;     // lr / (1 - beta1^t)
  float inv_sqrt_bc2;  // 1 / sqrt(1 - beta2^t)
  float eps_adam;
};

constexpr int kThreads = 256;             // threads per workgroup of every streaming kernel
constexpr int kMaxGridBlocks = 1 << 16;   // upper bound on workgroups per launch (partials buffer)

enum StateOp { kStateZero = 0, kStateCopy = 1 };

// How many workgroups of the fused AdamW kernel are resident on one CU at a time (its
// default grid is one resident wave of workgroups).
int adamw_blocks_per_cu(int dtype);

// Launchers (defined in gac_kernels.hip).  Each validates nothing: the host side has
// already checked shapes against the plan.  All return the launch's hipError_t.
// Pass 1 with the finalize step folded into its last-arriving workgroup.  The sums go to
// sums_out (if not null).  mode bit 1: decide and write the result record to dev_result and,
// if not null, also to host_result (host-mapped pinned memory).  dev_ticket is one zero
// word that the kernel leaves at zero.
hipError_t launch_reduce(int dtype, const Seg* dev_segs, int64_t n_chunks, int chunk_elems,
                         double* dev_partials, unsigned int* dev_ticket, int grid, double* sums_out,
                         gac_result* dev_result, gac_result* host_result, DecideParams p, int mode,
                         hipStream_t stream);

// Pass 1 of the snapshot form (p.cur set), two launches: the streaming kernel (the sums per
// chunk, and the raw gradient written to the state buffer that is not current, snap_delta bytes
// from the other) and a small kernel that adds the chunk sums in a fixed order and does the
// finalize step.  Working memory: a chunk counter and a ticket word (zero at launch, left at
// zero), 3 doubles per chunk, 3 doubles per group of chunks (snap_group_count of them).
struct SnapBuffers {
  unsigned long long* draw;
  double* chunk_sums;
  double* group_sums;
  unsigned int* ticket;
};
int64_t snap_group_count(int64_t n_chunks);
hipError_t launch_snap_reduce(int dtype, const Seg* dev_segs, int64_t n_chunks, int chunk_elems,
                              const SnapBuffers& b, int grid, double* sums_out, gac_result* dev_result,
                              gac_result* host_result, DecideParams p, int mode, int64_t snap_delta,
                              hipStream_t stream);

// The finalize step alone, on sums that come from elsewhere (device, 3 doubles): decides and
// writes the result record like the folded form.
hipError_t launch_finalize(const double* sums_in, double* sums_out, gac_result* dev_result,
                           gac_result* host_result, DecideParams p, hipStream_t stream);

// The pass-2 launchers take dev_work, a device counter that must be zero at launch (the
// finalize step leaves it so): their workgroups draw chunk indices from it.
hipError_t launch_apply(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                        int chunk_elems, const gac_result* dev_result, unsigned long long* dev_work,
                        int grid, hipStream_t stream);

// Table 3 statistics over ring entries of steps first_step .. last_step (1-based, at most
// hist_cap of them); writes *dev_out and, if not null, *host_out (host-mapped).
hipError_t launch_diag(const double* hist_c, const int32_t* hist_regime, int hist_cap,
                       int64_t first_step, int64_t last_step, double c_low, gac_diag* dev_out,
                       gac_diag* host_out, hipStream_t stream);

// Buffer-exchange pass 2: writes g' over the old state (Seg::b) in the projection regime only.
hipError_t launch_exchange(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                           int chunk_elems, const gac_result* dev_result,
                           unsigned long long* dev_work, int grid, hipStream_t stream);

// Pass 2 of the snapshot form: g <- scale_g g + coef_d d_old in place when the step projects or
// clips, nothing otherwise (the state was already written by pass 1).
hipError_t launch_snap_apply(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                             int chunk_elems, const gac_result* dev_result,
                             unsigned long long* dev_work, int32_t* dev_cur, int64_t snap_delta,
                             int grid, hipStream_t stream);

// The same traffic as the projecting apply pass with every value written back unchanged.
hipError_t launch_apply_probe(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                              int chunk_elems, unsigned long long* dev_work, int grid,
                              hipStream_t stream);
hipError_t launch_apply_adamw(int dtype, const Seg* dev_segs, const AdamSeg* dev_adam,
                              int n_tensors, int64_t n_chunks, int chunk_elems,
                              const gac_result* dev_result, unsigned long long* dev_work,
                              AdamScalars h, int grid, hipStream_t stream);

// Threshold pairs of one sweep, passed to the kernel by value.
struct SweepPairs {
  double c_low[64];
  double c_high[64];
};
hipError_t launch_sweep(const double* hist_c, const int32_t* hist_regime, int hist_cap,
                        int64_t first_step, int64_t last_step, const SweepPairs& pairs,
                        int n_pairs, int32_t* host_counts, hipStream_t stream);
// Set the device-side step counter (init / reset / import) or one 32-bit word (ticket counter,
// current-buffer flag); one-thread kernels rather than memsets so that they can sit in a
// captured graph.
hipError_t launch_set_step(int64_t* dev_step, int64_t value, hipStream_t stream);
hipError_t launch_set_word(uint32_t* dev_word, uint32_t value, hipStream_t stream);

hipError_t launch_state_op(int dtype, int op, const Seg* dev_segs, int64_t n_chunks,
                           int chunk_elems, int grid, hipStream_t stream);

// The entry point that allocates nothing keeps its device-side working memory in a static
// device array (one copy per GPU).  Limits of that array:
constexpr int kStaticMaxTensors = GAC_STATIC_MAX_TENSORS;
constexpr int kStaticMaxGrid = 1024;  // partial-sum slots
struct StaticScratch {
  unsigned int* ticket;
  unsigned long long* work;
  double* sums;
  gac_result* result;
  double* partials;
  Seg* segs;
};
// Device addresses of the parts of the static array on `device`, which must be the current
// device (the array's address is looked up once per device and kept).
hipError_t static_scratch(int device, StaticScratch* out);
size_t static_scratch_bytes();

// A batch of tensor-table entries small enough to travel as a kernel argument.
constexpr int kSegBatch = 96;
struct SegBatch {
  int32_t first, count;
  Seg e[kSegBatch];
};
// table[first + i] = e[i]; with ticket_to_clear not null also *ticket_to_clear = 0.
hipError_t launch_fill_segs(Seg* dev_table, const SegBatch& batch, unsigned int* ticket_to_clear,
                            hipStream_t stream);

}  // namespace gac
