/* gac.h - C ABI of the MI355X Gradient Alignment Control (GAC) step library.
 *
 * One call of gac_step() is one iteration of the body of Algorithm 1 of
 * "GAC: Stabilizing Asynchronous RL Training for LLMs via Gradient Alignment
 * Control" (arXiv 2603.01501) between "gradient is ready" and "optimizer
 * consumes it":
 *
 *   1. three inner products <g,d>, <g,g>, <d,d> over the whole list of
 *      parameter gradients g and the reference state d (Appendix A.1),
 *   2. c = <g,d> / (sqrt(<g,g><d,d>) + eps)                  (Eq. 1, App. A.1),
 *   3. regime: |c| <= c_low safe, |c| >= c_high violation (skip the update),
 *      otherwise projection                           (Section 4.2, Algorithm 1),
 *   4. projection: g <- beta g + (alpha - beta) <g,u> u in place, u = d/|d|,
 *      alpha = c_low/|c|, beta = 1                   (Eq. 2-4, Appendix A.2),
 *   5. d <- raw g of this step: the reference of the next step
 *      (Algorithm 1 initialises it to zero; Appendix A.2 "gradient snapshot").
 * Optional, both off by default: global-norm clipping of the gradient handed to the optimizer
 * folded into step 4 without another pass (Table 2 lists gradient clipping as on), and a
 * per-step record of c_t with the statistics of Table 3 (gac_diag_summary).
 *
 * General rules
 *   - Every pointer named "device" is GPU memory owned by the caller (for
 *     example PyTorch tensors); every other pointer is host memory.  Pointer
 *     LISTS (grad_ptrs, state_ptrs, ...) are host arrays of device pointers,
 *     one entry per tensor, copied during the call.
 *   - Tensors are contiguous and element-aligned; no further alignment is needed (views
 *     that start anywhere inside a flat buffer take the same vector path).  numel may be 0.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it.  A context is not thread-safe and its calls
 *     must be issued in stream order.
 *   - Functions return GAC_OK (0) or a negative GAC_ERR_* code; nothing throws
 *     or aborts across this boundary.  gac_strerror() names a code.
 *   - Results are deterministic: the same inputs, configuration and device give
 *     bit-identical sums, cosine and outputs on every call.
 *   - Magnitudes: the three sums are accumulated in fp64, but each product g*d, g*g, d*d is
 *     formed in fp32 first (exact for bf16 storage inside the fp32 exponent range).  Elements
 *     with magnitude roughly in [1e-18, 1e18] are therefore safe; squares of smaller ones
 *     underflow (a uniformly tiny gradient gives <g,g> = 0, c = 0, "safe") and squares of
 *     larger ones overflow (GAC_ERR_NONFINITE).  c is scale invariant (Appendix A.1), so a
 *     caller outside that range rescales g by a power of two.
 */
#ifndef GAC_H_
#define GAC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gac_ctx gac_ctx; /* opaque */

/* storage dtype of gradients and of the reference state */
enum { GAC_F32 = 0, GAC_BF16 = 1 };

/* regimes of Section 4.2 */
enum { GAC_SAFE = 0, GAC_PROJECT = 1, GAC_SKIP = 2 };

enum {
  GAC_OK = 0,
  GAC_ERR_INVALID_ARG = -1,    /* NULL where not allowed, negative sizes, bad dtype */
  GAC_ERR_BAD_THRESHOLDS = -2, /* violates 0 < c_low < c_high, eps < 0, beta < 0 */
  GAC_ERR_ALLOC = -3,          /* host or device allocation failed */
  GAC_ERR_HIP = -4,            /* a HIP runtime call failed; see gac_last_hip_error() */
  GAC_ERR_NONFINITE = -5,      /* a sum was inf/nan: nothing was modified (see gac_step) */
  GAC_ERR_UNIMPLEMENTED = -6,  /* this combination of entry point and configuration is not built */
  GAC_ERR_TOO_LARGE = -7       /* a size exceeds a fixed capacity of the library (gac_step_static) */
};

/* gac_config.flags */
#define GAC_FLAG_SNAPSHOT_IN_REDUCE 1u
/* Snapshot form, for callers that cannot swap buffers (gac_step_exchange) but whose steps are
 * mostly safe (Table 3 of the paper: 83-99 % of on-policy steps have |c_t| <= 0.05).  The library
 * keeps TWO state buffers; pass 1 writes the raw gradient into the spare one while it reduces
 * (Appendix A.2: the gradient snapshot), and the finalize step makes that buffer the current
 * reference state.  A step that neither projects nor clips then has no second pass: 3 N s
 * bytes instead of 4 N s.  A projecting step reads g and the old state and rewrites g
 * (3 N s + 3 N s, two mixed passes instead of one pure read pass and one mixed pass, so it
 * is slower than the default form).  Pass 1 of this form draws its chunks in order (which a
 * pass that also writes needs to be fast) and therefore keeps one partial sum per chunk,
 * combined in a fixed order: its results are the same bit for bit on every run and for every
 * grid_blocks, and equal to the default form's up to the rounding of the partial sums (the
 * two forms group the same products differently: ~1e-10 relative on the sums).  Costs N s bytes of device memory plus 24 bytes per chunk.  Needs a library-allocated state (state_ptrs =
 * NULL); works with gac_step and gac_reduce_local / gac_apply; gac_step_adamw and
 * gac_place_state return GAC_ERR_UNIMPLEMENTED on such a context. */

typedef struct gac_config {
  double c_low;   /* Section 4.2; paper default 0.05 (Appendix C, "GAC thresholds") */
  double c_high;  /* paper default 0.3; values > 1 mean "never skip" */
  double eps;     /* added to the cosine denominator, Appendix A.1; default 1e-8 */
  double beta;    /* gain of the orthogonal part, Eq. 3; the paper uses 1 (Appendix A.2) */
  int32_t dtype;  /* GAC_F32 or GAC_BF16 */
  int32_t n_tensors;
  const int64_t* numel;    /* host, n_tensors entries, copied by gac_init */
  void* const* state_ptrs; /* host list of device buffers for d, one per tensor, each
                              numel[j] elements of dtype, or NULL: the library allocates
                              (and frees in gac_destroy) one buffer for all of d */
  int32_t device;          /* HIP device ordinal; -1 = current device */
  uint32_t flags;          /* 0 or GAC_FLAG_SNAPSHOT_IN_REDUCE */
  int32_t chunk_elems;     /* tuning: elements per work item of a block; 0 = default.
                              Must be a positive multiple of 2048. */
  int32_t grid_blocks;     /* tuning: workgroups of the reduction launch (= number of partial
                              sums, so it is part of what fixes the result bits); 0 = default
                              (one per CU) */
  int32_t apply_blocks;    /* tuning: workgroups of the apply launch; 0 = default (7/8 of the CUs) */
  double max_grad_norm;    /* > 0: the gradient handed to the optimizer (g' when projected, g when
                              safe) is scaled by min(1, max_grad_norm / (its 2-norm + 1e-6)); the
                              norm comes from the three sums, so no extra pass.  0 = no clipping.
                              The reference state always keeps the raw, unclipped gradient. */
  int32_t history_capacity;/* steps of (c_t, regime) kept on the device for gac_history_read /
                              gac_diag_summary; 0 = default 1024; at most 4096 */
  int32_t reserved;        /* must be 0 */
} gac_config;

typedef struct gac_result {
  double dot;  /* <g,d> */
  double gg;   /* <g,g> */
  double dd;   /* <d,d> */
  double c;    /* cosine with eps; NaN if nonfinite */
  double alpha;/* c_low/|c| in the projection regime, else 1 */
  double coef; /* k in g' = beta g + k d;  (alpha-beta) <g,d>/<d,d> in the projection regime, else 0 */
  double grad_norm; /* 2-norm of the gradient GAC hands over, before clipping: |g'| when
                       projected (from the sums: beta^2<g,g> + 2 beta k <g,d> + k^2 <d,d>), else |g| */
  double clip_coef; /* factor applied by clipping, 1 if none (or clipping off, or GAC_SKIP) */
  double scale_g;   /* what pass 2 actually computes is  scale_g * g + coef_d * d : */
  double coef_d;    /*   scale_g = clip_coef * (beta if projected else 1), coef_d = clip_coef * coef */
  int32_t regime;    /* GAC_SAFE / GAC_PROJECT / GAC_SKIP */
  int32_t nonfinite; /* 1 if any sum was not finite */
  int32_t modified;  /* 1 if the gradient for the optimizer differs from the raw g (projected
                        and/or clipped): gac_step has overwritten g; gac_step_exchange has put it
                        into the returned buffers */
  int32_t reserved;
  int64_t step;      /* 1 for the first update after init/reset */
} gac_result;

/* Statistics of the recorded cosines, as in Table 3 of the paper (computed on the GPU). */
typedef struct gac_diag {
  int64_t first_step, last_step; /* range of recorded steps that was looked at (after burn-in) */
  int64_t n_values;              /* steps in that range with a finite c_t */
  int64_t n_nonfinite;           /* steps in that range whose sums were not finite */
  int64_t regime_count[3];       /* safe / projected / skipped steps in that range */
  double q90_abs_c;              /* 0.9-quantile of |c_t| (linear interpolation between order statistics) */
  double max_abs_c;
  double frac_le_c_low;          /* fraction of steps with |c_t| <= c_low (the current c_low) */
} gac_diag;

/* AdamW hyper-parameters; the paper's values are lr 1e-6, betas (0.9, 0.999),
 * eps 1e-8, weight decay 1e-2 (Table 2).  t_adam is the 1-based count of optimizer
 * steps actually taken, owned by the caller (a skipped update does not count). */
typedef struct gac_adamw_hyper {
  double lr, beta1, beta2, eps_adam, weight_decay;
  int64_t t_adam;
} gac_adamw_hyper;

/* Fills cfg with the paper's defaults (c_low 0.05, c_high 0.3, eps 1e-8, beta 1),
 * dtype GAC_BF16, no tensors, device -1. */
void gac_default_config(gac_config* cfg);

/* Algorithm 1, initialisation: creates a context for a fixed list of tensor sizes and
 * sets the reference state to zero (so the first step has c = 0 and is safe).
 * Thresholds are validated first (0 < c_low < c_high, eps >= 0, beta >= 0), before any
 * GPU call.  On failure *out is NULL. */
int gac_init(gac_ctx** out, const gac_config* cfg);

/* Frees everything the library allocated (never caller-provided state). NULL is allowed. */
void gac_destroy(gac_ctx* ctx);

/* One whole update (steps 1-5 above) on one GPU.
 *   grad_ptrs  host list of n_tensors device pointers to g (modified in place only in the
 *              projection regime).  May differ from call to call; sizes may not.  The
 *              gradient buffers must not overlap the state buffers: a pointer equal to the
 *              tensor's state pointer is rejected (GAC_ERR_INVALID_ARG), other overlaps are
 *              not detected.  The same holds for every entry point that takes grad_ptrs.
 *   host_out   NULL: fully asynchronous.  Otherwise the call waits until the regime is known
 *              (pass 2 may still be running) and fills *host_out; the caller skips its
 *              optimizer step if regime is GAC_SKIP.
 * With host_out == NULL and the same pointers as in the previous call, the call only launches
 * its kernels (two; three in the snapshot form; no copy, no host wait, no memset), so it can be captured into a HIP graph and
 * replayed: the step counter and the record of c_t live on the device and keep counting.
 * Thresholds and max_grad_norm are launch arguments and are frozen into a captured graph.
 * The state d becomes the raw g in all three regimes.  If a sum is not finite (a
 * convention of this library, the paper does not cover it): nonfinite = 1, regime =
 * GAC_SKIP, neither g nor d is touched, and the return value is GAC_ERR_NONFINITE when
 * host_out was given (otherwise GAC_OK, and the flag is in the device result). */
int gac_step(gac_ctx* ctx, void* const* grad_ptrs, void* hip_stream, gac_result* host_out);

/* The same update without the snapshot copy, for callers that can let buffers change hands.
 * Requires a context whose state buffers were provided by the caller (cfg->state_ptrs) and
 * host_out != NULL.  The g buffers passed in BECOME the reference state (the raw gradient is
 * the next reference: Algorithm 1, Appendix A.2) and the buffers that held the previous
 * reference state are returned in grad_ptrs:
 *   modified = 1 (projected, or clipped): the returned buffers hold the gradient for the
 *                optimizer (g' of Eq. 4, times the clip factor).  Traffic: 2 N s (statistics)
 *                + 3 N s instead of 6 N s.
 *   modified = 0 GAC_SAFE: the gradient to use is still in the buffers that were passed in;
 *                they now belong to the library and must only be read.  GAC_SKIP: no update.
 *                Nothing is moved at all (2 N s for the statistics only); the content of the
 *                returned buffers is unspecified.
 * In every regime the returned buffers are free for the caller's next gradient once the
 * optimizer is done with them.  On GAC_ERR_NONFINITE no buffer changes hands.  The call
 * returns when the regime is known; pass 2 may still be running on the stream. */
int gac_step_exchange(gac_ctx* ctx, void** grad_ptrs, void* hip_stream, gac_result* host_out);

/* Data-parallel form of the same update (Appendix A.1: each rank reduces its shard, one
 * all-reduce of three scalars, then each rank applies).  Phase 1 writes the rank-local
 * {<g,d>, <g,g>, <d,d>} to dev_sums3 (device, 3 doubles).  The caller sums them across
 * ranks (in a fixed order, if bit-reproducibility across runs is wanted). */
int gac_reduce_local(gac_ctx* ctx, void* const* grad_ptrs, void* hip_stream, double* dev_sums3);

/* Phase 2: takes the GLOBAL sums (device, 3 doubles), decides the regime and applies
 * steps 3-5 to the local shard.  gac_reduce_local + gac_apply on one rank with the same
 * sums is exactly gac_step. */
int gac_apply(gac_ctx* ctx, void* const* grad_ptrs, const double* dev_sums3, void* hip_stream,
              gac_result* host_out);

/* gac_step with the optimizer fused into the second pass: the projected gradient g' is
 * formed in registers and consumed by AdamW (decoupled weight decay; Table 2 names the
 * optimizer and its hyper-parameters) without being written back; g is left untouched.
 *   m <- b1 m + (1-b1) g';  v <- b2 v + (1-b2) g'^2;  p <- p - lr wd p;
 *   p <- p - lr (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps_adam)
 * master_p, m, v: host lists of device fp32 buffers (numel[j] each), updated in place.
 * p_lowp: optional host list of device buffers of the gradient dtype that receive the
 * rounded new parameters (NULL = none).  In the GAC_SKIP regime (and on nonfinite) the
 * optimizer state and parameters are not touched at all; d is still updated on SKIP. */
int gac_step_adamw(gac_ctx* ctx, void* const* grad_ptrs, float* const* master_p, float* const* m,
                   float* const* v, void* const* p_lowp, const gac_adamw_hyper* hyper,
                   void* hip_stream, gac_result* host_out);

/* gac_step for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No context: everything the step needs besides the caller's
 * buffers (tensor table, per-workgroup partial sums, ticket counter, sums, result record)
 * lives in a static device array inside the library, 57,856 bytes per GPU, held until the
 * process ends.  The call allocates nothing on host or device, calls no hipMalloc / hipFree,
 * copies nothing and waits for nothing: it only launches kernels on hip_stream (the tensor
 * table travels as kernel arguments, 96 tensors per launch), so it can be captured.
 *   cfg         thresholds, eps, beta, max_grad_norm, dtype, n_tensors, numel as for gac_init;
 *               state_ptrs is REQUIRED (the caller owns the reference state: numel[j] elements
 *               of dtype per tensor, zero before the first update); device as for gac_init;
 *               flags and history_capacity must be 0; chunk_elems, grid_blocks, apply_blocks
 *               are honoured (0 = the defaults of gac_init).
 *               Limits: n_tensors <= GAC_STATIC_MAX_TENSORS and grid_blocks <= 1024, else
 *               GAC_ERR_TOO_LARGE and nothing is launched.
 *   grad_ptrs   as for gac_step (modified in place in the projection regime)
 *   step        the number this update gets in the result record (the caller counts; the
 *               library keeps nothing between calls)
 *   result_out  NULL, or device-accessible memory (device memory, or host-mapped pinned memory)
 *               that receives the gac_result when the stream gets there
 * With the same configuration, device and inputs the gradient, the state and the result are
 * bit-identical to gac_step's.  All calls on one GPU share the one array: calls whose kernels
 * can overlap on that GPU (different streams, different threads) race and must be serialised
 * by the caller.  Nothing in the array has to survive from call to call (each call rewrites
 * the table and clears the counter it needs at zero). */
#define GAC_STATIC_MAX_TENSORS 1024
int gac_step_static(const gac_config* cfg, void* const* grad_ptrs, int64_t step, void* hip_stream,
                    gac_result* result_out);

/* Device address of the result of the most recent step, for callers that branch on the
 * GPU.  Valid until gac_destroy; overwritten by the next step. */
int gac_result_device(const gac_ctx* ctx, const gac_result** dev_ptr);

/* Copies the reference state d to / from caller buffers (host lists of device pointers,
 * numel[j] elements each).  Import also sets the step counter (checkpoint / resume). */
int gac_state_export(gac_ctx* ctx, void* const* dst_ptrs, int64_t* step_out, void* hip_stream);
int gac_state_import(gac_ctx* ctx, void* const* src_ptrs, int64_t step, void* hip_stream);

/* d <- 0 and step <- 0: back to the state right after gac_init. */
int gac_reset(gac_ctx* ctx, void* hip_stream);

/* State placement (for callers that let the library allocate the state; the paper does not
 * cover where buffers live).  Where the reference state sits in HBM relative to the gradients
 * changes the speed of both passes a little, in opposite directions: measured on MI355X, two
 * buffers in different thirds of the physical memory run the in-place pass ~3 % faster and the
 * read-only pass ~4 % slower than two buffers in the same third, so the whole step moves by
 * under 1 % (it was ~10 % before pass 2 drew its chunks in order).  Physical placement
 * cannot be requested, only observed, so this call measures.  It times the reduction pass and
 * a data-preserving probe of the in-place pass (the same loads, arithmetic and stores; every
 * value is written back unchanged) with the state where it is and with up to
 * max_candidates - 1 further allocations of the same size.  These are held until the end
 * (report->bytes_held_peak), with spacer allocations between them when the state is smaller
 * than 12 GiB, so that each lands at least 12 GiB deeper in memory than the one before.  The
 * search ends early once a location 3 % better than the first has been followed by two that
 * are no better, or after eight in a row without gain.  The state is then moved (contents
 * preserved bit for bit) to the location with the smallest sum of the two times if that is at
 * least 1 % better than where it was, everything else is freed, and the workgroup count of the
 * in-place pass is picked the same way (unless gac_config.apply_blocks fixed it).
 *   grad_ptrs        the gradient buffers the steps will use (contents preserved bit for bit;
 *                    nothing else may touch them during the call)
 *   max_candidates   1 .. GAC_MAX_PLACEMENT_CANDIDATES; 1 only tunes the workgroup count
 *   max_extra_bytes  cap on the temporary device memory; 0 = whatever is free less a 4 GiB
 *                    reserve.  The search stops quietly when memory runs out.
 *   report           optional; what was timed and what was chosen
 * A state the caller provided (gac_config.state_ptrs) cannot be moved: then max_candidates
 * must be 1 (else GAC_ERR_INVALID_ARG), and the call times the two passes where the buffers
 * are (report->probe_ms[0], reduce_ms[0]: what a caller needs to compare placements of its own)
 * and tunes the workgroup count.  Lists under 256 MiB are left alone (not bandwidth bound).
 * Set-up time call: allocates, waits for the stream, cannot be captured into a graph.  A
 * graph of steps captured earlier keeps working (it reads the pointer table, which this call
 * leaves on grad_ptrs and the final state) but keeps the workgroup count it was captured with.
 * The driver clears freed device memory in the background, which takes HBM bandwidth for a few
 * seconds after the call (measured: ~4 % on the reduction pass for ~2.5 s per 100 GB freed). */
#define GAC_MAX_PLACEMENT_CANDIDATES 16
typedef struct gac_placement {
  int32_t n_candidates; /* locations timed; index 0 is where the state was */
  int32_t chosen;       /* index of the location now in use */
  int32_t apply_blocks; /* workgroups of the in-place pass from now on */
  int32_t n_blocks_tried;
  double probe_ms[GAC_MAX_PLACEMENT_CANDIDATES];  /* in-place probe time per location */
  double reduce_ms[GAC_MAX_PLACEMENT_CANDIDATES]; /* reduction pass time per location */
  int32_t blocks_tried[4];
  double blocks_ms[4];  /* probe time at the chosen location per workgroup count */
  int64_t bytes_held_peak; /* most device memory the search held at one time beyond the state
                              itself (candidates and spacers), in bytes; all of it is freed again
                              except, after a move, what the old state occupied */
} gac_placement;
int gac_place_state(gac_ctx* ctx, void* const* grad_ptrs, int32_t max_candidates,
                    int64_t max_extra_bytes, void* hip_stream, gac_placement* report);

/* Replaces the thresholds (validated as in gac_init) for the following steps. */
int gac_set_thresholds(gac_ctx* ctx, double c_low, double c_high);

/* Copies the most recent recorded steps (oldest first, at most max_n) to host arrays: c_out
 * gets c_t (NaN for a non-finite step), regime_out the regime; either may be NULL.  n_out
 * receives the count and first_step_out the step number of the first entry.  Waits for the
 * stream.  Records start again after gac_reset / gac_state_import. */
int gac_history_read(gac_ctx* ctx, int64_t max_n, double* c_out, int32_t* regime_out,
                     int64_t* n_out, int64_t* first_step_out, void* hip_stream);

/* The statistics the paper uses to place its thresholds (Table 3: q0.9(|c_t|), max |c_t| and
 * Pr(|c_t| <= c_low) "over updates after step 50"), over the recorded steps with step number
 * > burn_in.  One small kernel on the stream; waits for it. */
int gac_diag_summary(gac_ctx* ctx, int64_t burn_in, gac_diag* out, void* hip_stream);

/* Threshold sweep over the record (the paper's Table 4 varies (c_low, c_high) around the
 * defaults; Section 4.2 gives the rule).  c_t is computed from the raw gradients before any
 * intervention (Appendix A.1), so on a given gradient sequence it does not depend on the
 * thresholds in force, and the regimes that any other pair would have chosen can be counted
 * from the record: for each pair i, counts[3*i + r] receives the number of recorded finite
 * steps with step number > burn_in that the pair (c_low[i], c_high[i]) puts in regime r
 * (GAC_SAFE, GAC_PROJECT, GAC_SKIP).  It says nothing about how training would have moved
 * under those thresholds.  c_low, c_high, counts: host arrays; 1 <= n_pairs <=
 * GAC_MAX_SWEEP_PAIRS; every pair must satisfy 0 < c_low < c_high (else
 * GAC_ERR_BAD_THRESHOLDS, nothing written).  One small kernel on the stream; waits for it. */
#define GAC_MAX_SWEEP_PAIRS 64
int gac_threshold_sweep(gac_ctx* ctx, int64_t burn_in, int32_t n_pairs, const double* c_low,
                        const double* c_high, int32_t* counts, void* hip_stream);

/* Host-only planning query (no GPU call): the number of work items the tensor list is cut
 * into (no item straddles two tensors) and the total element count.  chunk_elems = 0 uses
 * the default for the dtype. */
int gac_plan_query(const int64_t* numel, int32_t n_tensors, int32_t dtype, int32_t chunk_elems,
                   int64_t* n_chunks_out, int64_t* total_numel_out);

/* Kernel timing for benchmarks.  While enabled, each step records HIP events on its stream
 * around the reduction, the finalize and the apply kernels.  gac_profile_read waits for the
 * recorded events and returns the summed milliseconds per kernel and the number of steps
 * since the last read (which it then clears).  At most 1024 steps are kept.  The finalize
 * step runs inside the reduction kernel (its last workgroup to finish), so ms_finalize is
 * the empty interval between two events except for gac_apply, which has a finalize launch
 * of its own.  The events cost a few microseconds per step: keep them out of timed runs. */
int gac_profile_enable(gac_ctx* ctx, int32_t on);
int gac_profile_read(gac_ctx* ctx, double* ms_reduce, double* ms_finalize, double* ms_apply,
                     int32_t* n_steps);

const char* gac_strerror(int code);
/* Text of the last HIP error seen by this context (empty string if none).  With ctx = NULL:
 * the last HIP error of any context on the calling thread (for a failed gac_init). */
const char* gac_last_hip_error(const gac_ctx* ctx);
const char* gac_version(void);
/* SHA-256 (hex) of the sources this binary was built from, as the build recorded it ("" if it
 * did not); lets a loader refuse a binary that does not belong to the sources beside it. */
const char* gac_source_hash(void);

#ifdef __cplusplus
}
#endif
#endif /* GAC_H_ */
