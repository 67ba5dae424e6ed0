// HIP kernels of the GAC step for gfx950 (CDNA4, 64-wide wavefronts).
//
// The step is two streaming passes over the gradient list g and the reference state d:
//   pass 1 (reduce_kernel)   three inner products <g,d>, <g,g>, <d,d>      (Appendix A.1)
//     its last workgroup     cosine with eps, regime, alpha, coefficient    (Eq. 1, Sec. 4.2)
//   pass 2 (apply_kernel)    g <- beta g + k d in place and d <- raw g      (Eq. 4, App. A.2)
//          (apply_adamw_kernel: the same with AdamW consuming g' in registers, Table 2;
//           exchange_kernel: g' written over the old state, for callers that swap buffers;
//           snap_apply_kernel: g' alone, when pass 1 has already written the snapshot)
// Beside them: finalize_kernel (the scalar step alone, for sums that come from other ranks),
// state_kernel (zero / copy of the state), diag_kernel and sweep_kernel (the statistics of
// Table 3 and regime counts under other thresholds over the recorded c_t).
// Both passes are bound by HBM bandwidth (3 FMA per 2 loaded elements, 1 FMA per 4 moved
// elements), so there is no matrix-core work here; what matters is 16-byte accesses that
// coalesce to full cache lines, many loads in flight per wave, all CUs busy to the end, and
// workgroups that work on neighbouring parts of memory at the same time.
//
// Work distribution: the tensor list is cut into chunks (gac_internal.h: Seg).
// Pass 1: workgroup b of a G-wide persistent grid takes chunks b, b+G, b+2G, ...  The
// chunk -> workgroup map is static, every workgroup writes its own partial sums, and the last
// workgroup to finish adds them in a fixed order (lane j takes partials j, j+256, ...; then a
// fixed tree over lanes and waves), so results are bit-reproducible.  No floating-point
// atomics anywhere.
// Pass 2 is element-wise, so any assignment gives the same bits: its workgroups draw chunk
// indices in order from a device-wide counter (walk_tiles).
//
// Accumulation: products are formed and summed in fp32 over one group of at most
// GAC_REDUCE_UNROLL * 8 elements per lane (for bf16 inputs each product is exact in fp32), then the
// group sum is widened and accumulated in fp64 per lane; wave, workgroup and grid combines
// are fp64.

#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

#include "gac_internal.h"

namespace gac {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// Pointers read from the tensor table are generic; casting them to the global address
// space lets the compiler emit global_load/global_store instead of flat accesses.
#define GAC_GLOBAL __attribute__((address_space(1)))
// Tensors are only guaranteed element alignment (views into flat parameter buffers start
// anywhere), so the 16- and 8-byte accesses are declared with 2-byte alignment.  The target
// supports unaligned vector memory accesses, so the compiler still emits one
// global_load_dwordx4 / dwordx2 per access; aligned tensors lose nothing.
typedef u32x4 u32x4_ua __attribute__((aligned(2)));
typedef u32x2 u32x2_ua __attribute__((aligned(2)));
typedef GAC_GLOBAL u32x4_ua gvec;
typedef GAC_GLOBAL char gchar;
typedef GAC_GLOBAL float gfloat;
typedef GAC_GLOBAL uint32_t gu32;
typedef GAC_GLOBAL uint16_t gu16;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Tuning constants, chosen from A/B measurements on MI355X with the tensors held fixed.
// Both passes saturate HBM with FEW workgroups that each keep many 16-byte accesses in
// flight; more resident waves only add contention at the memory controllers.
// Pass 1 is a pure read stream: one 256-thread workgroup per CU, 8 x 16 B loads per array
// in flight per lane, non-temporal loads (7.0-7.2 TB/s; 6.7 with six workgroups per CU; 16 or
// 32 loads per array in flight are 1-2 % slower, and so is an explicit second register tile
// that loads ahead, which is what the passes that also write need).
// Pass 2 reads and writes the same lines: 512-thread workgroups that load a whole tile of each
// array and then store it, the next tile's loads issued before the stores, on 7/8 of the CUs
// (13/16 is 0.4 % slower, 3/4 1.8 %, all CUs 3.5 %), non-temporal loads and stores.  What the
// tile size has to hit is the length of one burst of stores of a workgroup, 64 KiB: the state
// copy and the buffer-exchange and snapshot forms write one array and take a 64 KiB chunk per
// tile (8 vectors per lane); the in-place projection writes two arrays and takes half a chunk
// of each (4 vectors per lane and array: 9.51 -> 9.04 ms on a 7.6B bf16 list; a quarter
// chunk 12.2 ms, and half-chunk tiles for the one-array kernels 7.5 against 6.9 ms).  256 x 16
// and 1024 x 4 tiles are within 3 % of 512 x 8.  The cache policy of the stores (plain, nt,
// sc1, sc0 sc1 and combinations) changes a write stream by under 2 %.
// The fused AdamW pass moves nine streams: 512-thread workgroups, one per CU (by register
// count), two register tiles of 4 quads per lane and array, the next one loading while the
// current one is stored: 35.4 ms on a 7.6B list against 37.7 ms for one tile of 8 quads
// (14B: 67.8 against 69.4 ms); two tiles of 2 quads 36.9 ms, 256-thread workgroups 35.9 ms.
#ifndef GAC_REDUCE_THREADS
#define GAC_REDUCE_THREADS 256
#endif
#ifndef GAC_REDUCE_UNROLL
#define GAC_REDUCE_UNROLL 8
#endif
#ifndef GAC_REDUCE_NT_LOAD
#define GAC_REDUCE_NT_LOAD 1
#endif
#ifndef GAC_APPLY_THREADS
#define GAC_APPLY_THREADS 512
#endif
#ifndef GAC_APPLY_UNROLL
#define GAC_APPLY_UNROLL 8
#endif
#ifndef GAC_APPLY_SPLIT
#define GAC_APPLY_SPLIT 2
#endif
#ifndef GAC_APPLY_NT_LOAD
#define GAC_APPLY_NT_LOAD 1
#endif
#ifndef GAC_APPLY_NT_STORE
#define GAC_APPLY_NT_STORE 1
#endif
#ifndef GAC_ADAMW_THREADS
#define GAC_ADAMW_THREADS 512
#endif
#ifndef GAC_ADAMW_NT_LOAD
#define GAC_ADAMW_NT_LOAD 1
#endif
#ifndef GAC_ADAMW_QUADS
#define GAC_ADAMW_QUADS 4
#endif

template <int DT> struct Elem;
template <> struct Elem<GAC_F32> {
  static constexpr int kSize = 4;
  static constexpr int kPerVec = 4;
};
template <> struct Elem<GAC_BF16> {
  static constexpr int kSize = 2;
  static constexpr int kPerVec = 8;
};

template <int NT = 0>
__device__ __forceinline__ u32x4 ld16(const gvec* p) {
  if constexpr (NT) {
    return __builtin_nontemporal_load(p);
  } else {
    return *p;
  }
}

template <int NT = 1>
__device__ __forceinline__ void st16(gvec* p, u32x4 v) {
  if constexpr (NT) {
    __builtin_nontemporal_store(v, p);
  } else {
    *p = v;
  }
}

// 16 raw bytes -> fp32 values.  bf16 is the upper half of a binary32, element 0 in the
// low half of word 0 (little endian).
template <int DT>
__device__ __forceinline__ void unpack(u32x4 v, float (&x)[Elem<DT>::kPerVec]) {
  if constexpr (DT == GAC_F32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(v[i]);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(v[i] << 16);
      x[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
  }
}

// fp32 -> bf16 pair, round to nearest even (the hardware conversion of gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

template <int DT>
__device__ __forceinline__ u32x4 pack(const float (&x)[Elem<DT>::kPerVec]) {
  u32x4 v;
  if constexpr (DT == GAC_F32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = __float_as_uint(x[i]);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
  }
  return v;
}

template <int DT>
__device__ __forceinline__ float load_elem(const gchar* p, int i) {
  if constexpr (DT == GAC_F32) {
    return reinterpret_cast<const gfloat*>(p)[i];
  } else {
    return __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const gu16*>(p)[i]) << 16);
  }
}

template <int DT>
__device__ __forceinline__ void store_elem(gchar* p, int i, float x) {
  if constexpr (DT == GAC_F32) {
    reinterpret_cast<gfloat*>(p)[i] = x;
  } else {
    reinterpret_cast<gu16*>(p)[i] = static_cast<uint16_t>(pack_bf16x2(x, 0.0f) & 0xffffu);
  }
}

template <int DT>
__device__ __forceinline__ void copy_elem(const gchar* src, gchar* dst, int i) {
  if constexpr (DT == GAC_F32) {
    reinterpret_cast<gu32*>(dst)[i] = reinterpret_cast<const gu32*>(src)[i];
  } else {
    reinterpret_cast<gu16*>(dst)[i] = reinterpret_cast<const gu16*>(src)[i];
  }
}

// One contiguous piece of one tensor.
struct Chunk {
  const gchar* a;
  gchar* b;
  int64_t elem_off;  // offset of the chunk inside its tensor, in elements
  int len;           // elements in this chunk (the last chunk of a tensor may be short)
  int tensor;
};

// Finds the tensor that owns global chunk c.  `t` is a cursor that only moves in the
// direction the caller walks the chunk order (forward: REVERSE = false).
template <bool REVERSE>
__device__ __forceinline__ Chunk locate(const Seg* __restrict__ segs, int& t, int64_t c,
                                        int chunk_elems, int esize) {
  if constexpr (REVERSE) {
    while (c < segs[t].first_chunk) --t;
  } else {
    while (c >= segs[t + 1].first_chunk) ++t;
  }
  const Seg s = segs[t];
  Chunk ch;
  ch.elem_off = (c - s.first_chunk) * static_cast<int64_t>(chunk_elems);
  const int64_t rest = s.numel - ch.elem_off;
  ch.len = rest < chunk_elems ? static_cast<int>(rest) : chunk_elems;
  ch.a = (const gchar*)(s.a) + ch.elem_off * esize;
  ch.b = (gchar*)(s.b) + ch.elem_off * esize;
  ch.tensor = t;
  return ch;
}

// A value that is the same in every lane (read from LDS, say), moved to scalar registers so
// that what depends on it (table lookups, loop control) is scalar work.
__device__ __forceinline__ int64_t uniform64(int64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(v) >> 32));
  return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
}

// One chunk of g and of d in registers: U vectors per lane and array.
template <int U>
struct PairTile {
  static constexpr int kU = U;
  u32x4 a[U], b[U];
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Sum of three per-lane doubles over the workgroup; the result is valid in thread 0.
template <int T>
__device__ __forceinline__ void block_sum3(double (&s)[3]) {
  __shared__ double sm[3][T / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    s[k] = wave_sum(s[k]);
    if (lane == 0) sm[k][wave] = s[k];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      double acc = sm[k][0];
#pragma unroll
      for (int w = 1; w < T / 64; ++w) acc += sm[k][w];
      s[k] = acc;
    }
  }
}

// ------------------------------------------------------------------ finalize

// Adds the per-workgroup partial sums in a fixed order: lane j < kThreads takes partials j,
// j + kThreads, ..., then a fixed tree over lanes and waves (lanes beyond kThreads, in a wider
// workgroup, add zeros, which changes no bit).  The result is valid in thread 0.
template <int T>
__device__ __forceinline__ void combine_partials(const double* __restrict__ partials, int n_partials,
                                                 double (&s)[3]) {
  static_assert(T >= kThreads, "the combine is defined over kThreads lanes");
  s[0] = s[1] = s[2] = 0.0;
  if (threadIdx.x < kThreads) {
    for (int j = threadIdx.x; j < n_partials; j += kThreads) {
      s[0] += partials[3 * j + 0];
      s[1] += partials[3 * j + 1];
      s[2] += partials[3 * j + 2];
    }
  }
  block_sum3<T>(s);
}

// One thread: cosine with eps, regime, alpha, coefficients, clipping, the record of c_t and
// the result (Appendix A.1, Section 4.2, Algorithm 1, Appendix A.2).
__device__ __forceinline__ void decide_and_record(const double (&s)[3], const DecideParams& p,
                                                  gac_result* __restrict__ res,
                                                  gac_result* __restrict__ host_res) {
  const double s_gd = s[0], s_gg = s[1], s_dd = s[2];
  int64_t step;
  if (p.step != nullptr) {
    step = *p.step + 1;  // only this one thread of the launch touches the counter
    *p.step = step;
  } else {
    step = p.step_value;
  }
  gac_result r;
  r.dot = s_gd;
  r.gg = s_gg;
  r.dd = s_dd;
  r.alpha = 1.0;
  r.coef = 0.0;
  r.grad_norm = 0.0;
  r.clip_coef = 1.0;
  r.scale_g = 1.0;
  r.coef_d = 0.0;
  r.nonfinite = 0;
  r.modified = 0;
  r.reserved = 0;
  r.step = step;
  if (!(isfinite(s_gd) && isfinite(s_gg) && isfinite(s_dd))) {
    r.c = __longlong_as_double(0x7ff8000000000000LL);
    r.regime = GAC_SKIP;
    r.nonfinite = 1;
  } else {
    // Appendix A.1: eps is added to the square root of the product of the squared norms.
    const double c = s_gd / (sqrt(s_gg * s_dd) + p.eps);
    const double mag = fabs(c);
    r.c = c;
    double norm_sq = s_gg;  // squared norm of the gradient handed to the optimizer
    if (mag <= p.c_low) {   // Algorithm 1 tests the safe branch first
      r.regime = GAC_SAFE;
    } else if (mag >= p.c_high) {
      r.regime = GAC_SKIP;
    } else {
      r.regime = GAC_PROJECT;
      r.alpha = p.c_low / mag;
      // <g,u> u = (<g,d>/<d,d>) d, so g' = beta g + (alpha - beta)(<g,d>/<d,d>) d.
      // |c| > c_low > 0 implies <d,d> > 0.
      r.coef = (r.alpha - p.beta) * (s_gd / s_dd);
      r.scale_g = p.beta;
      r.coef_d = r.coef;
      r.modified = 1;
      // |beta g + k d|^2 from the three sums: no further pass over the data
      norm_sq = p.beta * p.beta * s_gg + 2.0 * p.beta * r.coef * s_gd + r.coef * r.coef * s_dd;
    }
    r.grad_norm = sqrt(norm_sq > 0.0 ? norm_sq : 0.0);
    if (p.max_grad_norm > 0.0 && r.regime != GAC_SKIP) {
      const double clip = p.max_grad_norm / (r.grad_norm + 1e-6);
      if (clip < 1.0) {
        r.clip_coef = clip;
        r.scale_g *= clip;
        r.coef_d *= clip;
        r.modified = 1;
      }
    }
  }
  if (p.hist_c != nullptr) {
    const int slot = static_cast<int>((step - 1) % p.hist_cap);
    p.hist_c[slot] = r.c;
    p.hist_regime[slot] = r.nonfinite ? -1 : r.regime;
  }
  // The snapshot form keeps two state buffers; a finite step makes the one that pass 1 has
  // just filled with the raw gradient the current one.
  if (p.cur != nullptr && !r.nonfinite) *p.cur ^= 1;
  *res = r;
  // Optional second copy straight into host-mapped pinned memory: the host then learns the
  // regime by waiting on an event after this kernel, with no copy command in the stream.
  if (host_res != nullptr) *host_res = r;
}

// What follows the sums, for the kernel that has them.
//   mode bit 0: the sums come from the per-workgroup partials (else from sums_in);
//   mode bit 1: evaluate the cosine and the regime and write the result record.
struct FinalArgs {
  const double* sums_in;
  double* sums_out;      // may be null
  gac_result* res;
  gac_result* host_res;  // may be null
  DecideParams p;
  int mode;
};

// Thread 0 holds the sums.
__device__ __forceinline__ void finish(const double (&s)[3], const FinalArgs& f) {
  if (f.p.work != nullptr) *f.p.work = 0ull;  // pass 2 draws its chunks from zero
  if (f.sums_out != nullptr) {
    f.sums_out[0] = s[0];
    f.sums_out[1] = s[1];
    f.sums_out[2] = s[2];
  }
  if (f.mode & 2) decide_and_record(s, f.p, f.res, f.host_res);
}

// Stand-alone form, for sums that come from elsewhere (the data-parallel phase 2).
__global__ __launch_bounds__(kThreads) void finalize_kernel(const double* __restrict__ partials,
                                                            int n_partials, FinalArgs f) {
  double s[3] = {0.0, 0.0, 0.0};
  if (f.mode & 1) {
    combine_partials<kThreads>(partials, n_partials, s);
  } else if (threadIdx.x == 0) {
    s[0] = f.sums_in[0];
    s[1] = f.sums_in[1];
    s[2] = f.sums_in[2];
  }
  if (threadIdx.x == 0) finish(s, f);
}

// ------------------------------------------------------------------ pass 1: reduction

template <int DT>
__device__ __forceinline__ void dot3(u32x4 a, u32x4 b, float& gd, float& gg, float& dd) {
  constexpr int N = Elem<DT>::kPerVec;
  float x[N], y[N];
  unpack<DT>(a, x);
  unpack<DT>(b, y);
#pragma unroll
  for (int e = 0; e < N; ++e) {
    gd = fmaf(x[e], y[e], gd);
    gg = fmaf(x[e], x[e], gg);
    dd = fmaf(y[e], y[e], dd);
  }
}

// The snapshot form keeps two buffers per state tensor, `delta` bytes apart (Seg::b is buffer
// 0); *cur says which one holds the reference state.  Pass 1 then also writes the raw gradient
// into the other one, which the finalize step makes current, so that a step that neither
// projects nor clips needs no second pass at all (3 N s bytes instead of 4 N s).
struct SnapArgs {
  int32_t* cur;
  int64_t delta;
};

// Pass 1.  Besides its partial sums every workgroup takes a ticket (an integer atomic, so the
// order of arrival changes nothing in the result); the one that draws the last ticket knows
// that all partial sums have been written, adds them in the fixed order and does what follows
// the sums (FinalArgs), so the step needs no separate finalize launch.  It also puts the
// ticket counter back to zero for the next launch.
//
// The chunk -> workgroup map is a static stride on purpose: for this pure read stream it
// measured 10 % FASTER than chunks drawn in order (4.24 ms against 4.75-4.94 ms on the
// 7.6B-parameter bf16 list), the opposite of the passes that also write.
template <int DT, int T, int U>
__global__ __launch_bounds__(T) void reduce_kernel(const Seg* __restrict__ segs,
                                                          int64_t n_chunks, int chunk_elems,
                                                          double* __restrict__ partials,
                                                          unsigned int* __restrict__ ticket,
                                                          FinalArgs fin) {
  constexpr int N = Elem<DT>::kPerVec;
  const int tid = threadIdx.x;
  double acc[3] = {0.0, 0.0, 0.0};
  int t = 0;
  int64_t c = blockIdx.x;
  bool more = c < n_chunks;
  Chunk next = {};
  if (more) next = locate<false>(segs, t, c, chunk_elems, Elem<DT>::kSize);
  while (more) {
    const Chunk ch = next;
    // Look up the following chunk now: its dependent scalar loads from the tensor table
    // then overlap this chunk's streaming instead of stalling the workgroup between chunks.
    c += gridDim.x;
    more = c < n_chunks;
    if (more) next = locate<false>(segs, t, c, chunk_elems, Elem<DT>::kSize);
    {
      const gvec* __restrict__ gv = reinterpret_cast<const gvec*>(ch.a);
      const gvec* __restrict__ dv = reinterpret_cast<const gvec*>(ch.b);
      const int nvec = ch.len / N;
      int i = tid;
      for (; i + (U - 1) * T < nvec; i += U * T) {
        u32x4 a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = ld16<GAC_REDUCE_NT_LOAD>(gv + i + u * T);
#pragma unroll
        for (int u = 0; u < U; ++u) b[u] = ld16<GAC_REDUCE_NT_LOAD>(dv + i + u * T);
        float gd = 0.f, gg = 0.f, dd = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float pgd = 0.f, pgg = 0.f, pdd = 0.f;
          dot3<DT>(a[u], b[u], pgd, pgg, pdd);
          gd += pgd;
          gg += pgg;
          dd += pdd;
        }
        acc[0] += static_cast<double>(gd);
        acc[1] += static_cast<double>(gg);
        acc[2] += static_cast<double>(dd);
      }
      for (; i < nvec; i += T) {
        float gd = 0.f, gg = 0.f, dd = 0.f;
        dot3<DT>(ld16<GAC_REDUCE_NT_LOAD>(gv + i), ld16<GAC_REDUCE_NT_LOAD>(dv + i), gd, gg, dd);
        acc[0] += static_cast<double>(gd);
        acc[1] += static_cast<double>(gg);
        acc[2] += static_cast<double>(dd);
      }
      const int e = nvec * N + tid;  // at most N-1 leftover elements
      if (e < ch.len) {
        const float x = load_elem<DT>(ch.a, e), y = load_elem<DT>(ch.b, e);
        acc[0] += static_cast<double>(x * y);
        acc[1] += static_cast<double>(x * x);
        acc[2] += static_cast<double>(y * y);
      }
    }
  }
  block_sum3<T>(acc);
  __shared__ int last_arrival;
  if (tid == 0) {
    partials[3 * blockIdx.x + 0] = acc[0];
    partials[3 * blockIdx.x + 1] = acc[1];
    partials[3 * blockIdx.x + 2] = acc[2];
    __threadfence();  // the partial sums are visible device-wide before the ticket is drawn
    last_arrival = atomicAdd(ticket, 1u) == gridDim.x - 1;
  }
  __syncthreads();
  if (!last_arrival) return;
  __threadfence();  // every other workgroup's partial sums are read from memory, not from a stale cache line
  double s[3];
  combine_partials<T>(partials, static_cast<int>(gridDim.x), s);
  if (tid == 0) {
    finish(s, fin);
    *ticket = 0u;
  }
}

// Pass 1 of the snapshot form: the three sums AND the raw gradient stored into the spare state
// buffer (2 N s read, N s written).  A pass that also writes is fastest with its chunks drawn
// in order (see walk_tiles; here 7.9 -> 6.9 ms against the static stride), so the sums cannot
// be per-workgroup partials: which workgroup takes which chunk is not reproducible.  Instead
// every CHUNK gets its own partial sums, computed by a tree that depends on nothing but the
// chunk (per lane two fp32 group sums of 8 vectors each, widened and added; a wave reduction;
// the four waves in order), and snap_combine_kernel adds them in two fixed levels.  The result
// therefore does not depend on the grid or on timing, only on the data, the chunk size and
// this tree.  (Publishing the chunk sums and combining them inside this kernel needs a
// device-wide fence per chunk, which waits for the chunk's stores to drain: 18.7 ms.)
struct SnapWork {
  unsigned long long* draw;   // chunk counter of this pass (zero at launch; the combine kernel zeroes it)
  double* chunk_sums;         // 3 doubles per chunk
  double* group_sums;         // 3 doubles per group of kSnapGroup chunks
  unsigned int* ticket;       // arrival counter of the combine kernel's workgroups (left at zero)
};
constexpr int kSnapGroup = 256;
constexpr int kSnapThreads = 256;  // one wave per SIMD; the whole chunk in registers, twice
constexpr int kSnapVecs = 16;      // vectors per lane and array of a whole chunk

template <int DT>
__global__ __launch_bounds__(kSnapThreads) void snap_reduce_kernel(const Seg* __restrict__ segs,
                                                                   int64_t n_chunks, int chunk_elems,
                                                                   SnapWork w, SnapArgs snap) {
  constexpr int N = Elem<DT>::kPerVec;
  constexpr int T = kSnapThreads, U = kSnapVecs, G = 8;  // G vectors per fp32 group, as in reduce_kernel
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool second = *snap.cur != 0;
  const int64_t d_off = second ? snap.delta : 0, spare_off = second ? 0 : snap.delta;

  __shared__ unsigned long long drawn[2];
  __shared__ double wave_part[2][3][T / 64];
  typedef PairTile<U> Tile;
  auto whole = [&](const Chunk& ch) { return ch.len == T * U * N; };
  auto draw = [&](int slot) {
    if (tid == 0) drawn[slot] = gridDim.x + atomicAdd(w.draw, 1ull);
  };
  auto load_tile = [&](const Chunk& ch, Tile& tl) {
    const gvec* gv = reinterpret_cast<const gvec*>(ch.a) + tid;
    const gvec* dv = reinterpret_cast<const gvec*>(ch.b + d_off) + tid;
#pragma unroll
    for (int u = 0; u < U; ++u) tl.a[u] = ld16<GAC_REDUCE_NT_LOAD>(gv + u * T);
#pragma unroll
    for (int u = 0; u < U; ++u) tl.b[u] = ld16<GAC_REDUCE_NT_LOAD>(dv + u * T);
  };
  // per-lane contribution of one chunk (and the snapshot stores)
  auto whole_chunk = [&](const Chunk& ch, const Tile& tl, double (&v)[3]) {
    gvec* sv = reinterpret_cast<gvec*>(ch.b + spare_off) + tid;
#pragma unroll
    for (int u = 0; u < U; ++u) st16<1>(sv + u * T, tl.a[u]);
    v[0] = v[1] = v[2] = 0.0;
#pragma unroll
    for (int grp = 0; grp < U / G; ++grp) {
      float gd = 0.f, gg = 0.f, dd = 0.f;
#pragma unroll
      for (int u = 0; u < G; ++u) {
        float pgd = 0.f, pgg = 0.f, pdd = 0.f;
        dot3<DT>(tl.a[grp * G + u], tl.b[grp * G + u], pgd, pgg, pdd);
        gd += pgd;
        gg += pgg;
        dd += pdd;
      }
      v[0] += static_cast<double>(gd);
      v[1] += static_cast<double>(gg);
      v[2] += static_cast<double>(dd);
    }
  };
  auto ragged_chunk = [&](const Chunk& ch, double (&v)[3]) {  // a tensor's tail, or another chunk size
    const gvec* gv = reinterpret_cast<const gvec*>(ch.a);
    const gvec* dv = reinterpret_cast<const gvec*>(ch.b + d_off);
    gvec* sv = reinterpret_cast<gvec*>(ch.b + spare_off);
    v[0] = v[1] = v[2] = 0.0;
    const int nvec = ch.len / N;
    for (int i = tid; i < nvec; i += T) {
      float gd = 0.f, gg = 0.f, dd = 0.f;
      const u32x4 a = ld16<GAC_REDUCE_NT_LOAD>(gv + i);
      dot3<DT>(a, ld16<GAC_REDUCE_NT_LOAD>(dv + i), gd, gg, dd);
      st16<1>(sv + i, a);
      v[0] += static_cast<double>(gd);
      v[1] += static_cast<double>(gg);
      v[2] += static_cast<double>(dd);
    }
    const int e = nvec * N + tid;  // at most N-1 leftover elements
    if (e < ch.len) {
      const float x = load_elem<DT>(ch.a, e), y = load_elem<DT>(ch.b + d_off, e);
      copy_elem<DT>(ch.a, ch.b + spare_off, e);
      v[0] += static_cast<double>(x * y);
      v[1] += static_cast<double>(x * x);
      v[2] += static_cast<double>(y * y);
    }
  };

  int t = 0;
  int64_t cr = blockIdx.x;
  if (cr >= n_chunks) return;
  draw(0);
  Chunk cur = locate<false>(segs, t, cr, chunk_elems, Elem<DT>::kSize);
  bool cur_whole = whole(cur);
  Tile tc = {};
  if (cur_whole) load_tile(cur, tc);
  int slot = 0;  // parity of the iteration: which half of the LDS hand-over buffers is written now
  for (;;) {
    // (1) this chunk's per-lane sums and its snapshot stores
    double v[3];
    if (cur_whole) {
      whole_chunk(cur, tc, v);
    } else {
      ragged_chunk(cur, v);
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      v[k] = wave_sum(v[k]);
      if (lane == 0) wave_part[slot][k][wave] = v[k];
    }
    __syncthreads();  // the wave sums and the index drawn one iteration ago are visible
    const int64_t this_chunk = cr;
    cr = uniform64(static_cast<int64_t>(drawn[slot]));
    const bool more = cr < n_chunks;
    // (2) the next chunk's loads go out before anything else
    Chunk next = cur;
    bool next_whole = false;
    Tile tn = {};
    if (more) {
      draw(slot ^ 1);
      next = locate<false>(segs, t, cr, chunk_elems, Elem<DT>::kSize);
      next_whole = whole(next);
      if (next_whole) load_tile(next, tn);
    }
    // (3) lane 0 adds the four waves in order and stores this chunk's sums
    if (tid == 0) {
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        double p = wave_part[slot][k][0];
#pragma unroll
        for (int x = 1; x < T / 64; ++x) p += wave_part[slot][k][x];
        w.chunk_sums[3 * this_chunk + k] = p;
      }
    }
    if (!more) break;
    cur = next;
    cur_whole = next_whole;
    tc = tn;
    slot ^= 1;
  }
}

// The chunk sums of snap_reduce_kernel, added in two fixed levels: workgroup s takes groups s,
// s + gridDim.x, ... of kSnapGroup consecutive chunks each (lane j the group's chunk j, then
// the fixed tree of block_sum3); the last workgroup to finish adds the group sums in index
// order and does the finalize step.  An empty list has no groups and its sums are zero.
__global__ __launch_bounds__(kThreads) void snap_combine_kernel(int64_t n_chunks, SnapWork w,
                                                                FinalArgs fin) {
  static_assert(kSnapGroup == kThreads, "one lane per chunk of a group");
  const int tid = threadIdx.x;
  const int64_t n_groups = (n_chunks + kSnapGroup - 1) / kSnapGroup;
  for (int64_t grp = blockIdx.x; grp < n_groups; grp += gridDim.x) {
    const int64_t first = grp * kSnapGroup;
    const int64_t count = n_chunks - first < kSnapGroup ? n_chunks - first : kSnapGroup;
    double s[3] = {0.0, 0.0, 0.0};
    if (tid < count) {
      s[0] = w.chunk_sums[3 * (first + tid) + 0];
      s[1] = w.chunk_sums[3 * (first + tid) + 1];
      s[2] = w.chunk_sums[3 * (first + tid) + 2];
    }
    block_sum3<kThreads>(s);
    if (tid == 0) {
      w.group_sums[3 * grp + 0] = s[0];
      w.group_sums[3 * grp + 1] = s[1];
      w.group_sums[3 * grp + 2] = s[2];
    }
    __syncthreads();  // block_sum3's LDS is free again
  }
  __shared__ int last_arrival;
  if (tid == 0) {
    __threadfence();
    last_arrival = atomicAdd(w.ticket, 1u) == gridDim.x - 1;
  }
  __syncthreads();
  if (!last_arrival) return;
  __threadfence();
  double g3[3];
  combine_partials<kThreads>(w.group_sums, static_cast<int>(n_groups), g3);
  if (tid == 0) {
    finish(g3, fin);
    *w.ticket = 0u;
    *w.draw = 0ull;
  }
}

// ------------------------------------------------------------------ pass 2: apply

template <int DT>
__device__ __forceinline__ u32x4 project_vec(u32x4 a, u32x4 b, float k, float beta) {
  constexpr int N = Elem<DT>::kPerVec;
  float x[N], y[N];
  unpack<DT>(a, x);
  unpack<DT>(b, y);
#pragma unroll
  for (int e = 0; e < N; ++e) x[e] = fmaf(k, y[e], beta * x[e]);
  return pack<DT>(x);
}

// Placement probe: the projected vector is computed like in a real step (with k = 0 and
// beta = 1 it equals g unless d holds a non-finite value) and g's own bits are stored
// whenever the two differ, so the probe does the arithmetic of the pass and changes nothing.
__device__ __forceinline__ u32x4 same_or(u32x4 computed, u32x4 original) {
  u32x4 out;
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = computed[i] == original[i] ? computed[i] : original[i];
  return out;
}

// A chunk that is not a whole tile (the tail of a tensor, or a non-default chunk size).
template <int DT, int T, int U, bool PROBE>
__device__ __forceinline__ void apply_chunk_generic(const Chunk& ch, bool project, float k,
                                                    float beta) {
  constexpr int N = Elem<DT>::kPerVec;
  const int tid = threadIdx.x;
  gchar* ga = const_cast<gchar*>(ch.a);
  gvec* gv = reinterpret_cast<gvec*>(ga);
  gvec* dv = reinterpret_cast<gvec*>(ch.b);
  const int nvec = ch.len / N;
  if (project) {
    for (int i = tid; i < nvec; i += T) {
      const u32x4 a = ld16<GAC_APPLY_NT_LOAD>(gv + i), b = ld16<GAC_APPLY_NT_LOAD>(dv + i);
      const u32x4 r = project_vec<DT>(a, b, k, beta);
      st16<GAC_APPLY_NT_STORE>(gv + i, PROBE ? same_or(r, a) : r);
      st16<GAC_APPLY_NT_STORE>(dv + i, PROBE ? b : a);
    }
    const int e = nvec * N + tid;  // at most N-1 leftover elements
    if (!PROBE && e < ch.len) {
      const float x = load_elem<DT>(ch.a, e), y = load_elem<DT>(ch.b, e);
      copy_elem<DT>(ch.a, ch.b, e);
      store_elem<DT>(ga, e, fmaf(k, y, beta * x));
    }
  } else {
    for (int i = tid; i < nvec; i += T) st16<GAC_APPLY_NT_STORE>(dv + i, ld16<GAC_APPLY_NT_LOAD>(gv + i));
    const int e = nvec * N + tid;
    if (e < ch.len) copy_elem<DT>(ch.a, ch.b, e);
  }
}

// The traversal shared by the pass-2 kernels.  A workgroup of T lanes owns one unit of work
// at a time: a chunk, or one of the SPLIT equal parts of a chunk.  A "whole tile" is a unit of
// exactly T*U vectors per array (the default chunk size, or its SPLIT-th part): each lane then
// holds U vectors of each array in registers, so the whole unit is read before any of it is
// written, and the loads of the workgroup's NEXT whole tile are issued before the current one
// is computed and stored (two register tiles), which keeps reads in flight during the
// arithmetic and the stores.  Other units (tensor tails, non-default chunk sizes) go to
// `generic`.
//
// Which workgroup takes which unit is decided while the kernel runs: workgroup b starts with
// unit b and draws every further one from a device-wide counter (*work, zero at launch; the
// finalize step resets it).  Pass 2 is element-wise, so the assignment changes no bit of the
// result, only who is idle at the end: with a static stride the workgroups of half the XCDs
// finished 0.5-6 % later than the others (measured on MI355X: they see a slower path to
// memory, and which half depends on the launch shape), and the kernel lasted as long as the
// slowest.  The index is fetched one chunk ahead by lane 0 and handed to the other lanes
// through LDS, one barrier per chunk.
//
// Chunks are walked from the end of the list towards its start (the reduction pass has just
// streamed the list front to back, so its last chunks would be the ones still cached).  With
// the non-temporal loads of pass 1 this measured no different from a forward walk on 2-3 GB
// lists; it is kept because it costs nothing.
template <int DT, int T, int U, typename Tile, int SPLIT = 1, typename Load, typename Store, typename Generic>
__device__ __forceinline__ void walk_tiles(const Seg* __restrict__ segs, int n_tensors,
                                           int64_t n_chunks_whole, int chunk_elems,
                                           unsigned long long* __restrict__ work, Load load_tile,
                                           Store store_tile, Generic generic) {
  constexpr int N = Elem<DT>::kPerVec;
  __shared__ unsigned long long drawn[2];
  auto whole = [&](const Chunk& ch) { return ch.len == T * U * N; };
  // lane 0 draws the next index into drawn[slot]; the others read it after the next barrier
  auto draw = [&](int slot) {
    if (threadIdx.x == 0) drawn[slot] = gridDim.x + atomicAdd(work, 1ull);
  };
  // The unit of work is 1/SPLIT of a chunk (SPLIT = 1: the chunk itself); units are numbered
  // like the chunks, the parts of one chunk one after the other.
  const int64_t n_chunks = n_chunks_whole * SPLIT;
  const int part = chunk_elems / SPLIT;  // chunk_elems is a multiple of 2048 elements
  auto locate_unit = [&](int& cursor, int64_t unit) {
    Chunk ch = locate<true>(segs, cursor, unit / SPLIT, chunk_elems, Elem<DT>::kSize);
    if constexpr (SPLIT > 1) {
      const int off = static_cast<int>(unit % SPLIT) * part;
      const int rest = ch.len - off;
      ch.len = rest < 0 ? 0 : (rest < part ? rest : part);  // a short chunk leaves late parts empty
      ch.a += static_cast<int64_t>(off) * Elem<DT>::kSize;
      ch.b += static_cast<int64_t>(off) * Elem<DT>::kSize;
      ch.elem_off += off;
    }
    return ch;
  };
  int t = n_tensors - 1;
  int64_t cr = blockIdx.x;
  if (cr >= n_chunks) return;
  draw(0);
  Chunk cur = locate_unit(t, n_chunks - 1 - cr);
  bool cur_whole = whole(cur);
  Tile tc = {};
  if (cur_whole) load_tile(cur, tc);
  __syncthreads();
  cr = uniform64(static_cast<int64_t>(drawn[0]));
  int slot = 1;
  for (;;) {
    const bool more = cr < n_chunks;
    Chunk next = cur;
    bool next_whole = false;
    Tile tn = {};
    if (more) {
      draw(slot);  // the index after this one: its latency hides behind this tile's traffic
      next = locate_unit(t, n_chunks - 1 - cr);
      next_whole = whole(next);
      if (next_whole) load_tile(next, tn);
    }
    if (cur_whole) {
      store_tile(cur, tc);
    } else {
      generic(cur);
    }
    if (!more) break;
    __syncthreads();
    cr = uniform64(static_cast<int64_t>(drawn[slot]));
    slot ^= 1;
    cur = next;
    cur_whole = next_whole;
    tc = tn;
  }
}

// Pass 2, in place: g <- scale_g g + coef_d d where the step projects and/or clips, d <- raw g.
//
// PROBE = true is the placement probe: the same loads, arithmetic and stores, but every value
// is written back where it came from (g <- g, d <- d), so nothing changes; it is timed to
// compare candidate locations of the state (gac_place_state).
template <int DT, int T, int U, bool PROBE>
__global__ __launch_bounds__(T) void apply_kernel(const Seg* __restrict__ segs,
                                                         int n_tensors, int64_t n_chunks,
                                                         int chunk_elems,
                                                         const gac_result* __restrict__ res,
                                                         unsigned long long* __restrict__ work,
                                                         float probe_k, float probe_beta) {
  if (!PROBE && res->nonfinite) return;  // convention: a non-finite step modifies nothing
  // g <- scale_g * g + coef_d * d when the step projects and/or clips, else g stays
  const bool project = PROBE || res->modified != 0;
  const float k = PROBE ? probe_k : static_cast<float>(res->coef_d);
  const float beta = PROBE ? probe_beta : static_cast<float>(res->scale_g);
  const int tid = threadIdx.x;

  auto generic = [&](const Chunk& ch) { apply_chunk_generic<DT, T, U, PROBE>(ch, project, k, beta); };
  if (project) {
    // Two arrays are read and two written: the tile is a part of a chunk, so that one burst of
    // stores of a workgroup is as long as in the copy below (tile shapes: see the tuning notes).
    constexpr int S = GAC_APPLY_SPLIT, UP = U / S;
    static_assert(U % S == 0 && UP >= 1, "the projecting tile is a whole fraction of the chunk tile");
    typedef PairTile<UP> Tile;
    auto load_tile = [&](const Chunk& ch, Tile& tl) {
      const gvec* gv = reinterpret_cast<const gvec*>(ch.a) + tid;
      const gvec* dv = reinterpret_cast<const gvec*>(ch.b) + tid;
#pragma unroll
      for (int u = 0; u < UP; ++u) tl.a[u] = ld16<GAC_APPLY_NT_LOAD>(gv + u * T);
#pragma unroll
      for (int u = 0; u < UP; ++u) tl.b[u] = ld16<GAC_APPLY_NT_LOAD>(dv + u * T);
    };
    auto store_tile = [&](const Chunk& ch, const Tile& tl) {
      gvec* gv = reinterpret_cast<gvec*>(const_cast<gchar*>(ch.a)) + tid;
      gvec* dv = reinterpret_cast<gvec*>(ch.b) + tid;
#pragma unroll
      for (int u = 0; u < UP; ++u) {
        const u32x4 r = project_vec<DT>(tl.a[u], tl.b[u], k, beta);
        st16<GAC_APPLY_NT_STORE>(gv + u * T, PROBE ? same_or(r, tl.a[u]) : r);
        st16<GAC_APPLY_NT_STORE>(dv + u * T, PROBE ? tl.b[u] : tl.a[u]);
      }
    };
    walk_tiles<DT, T, UP, Tile, S>(segs, n_tensors, n_chunks, chunk_elems, work, load_tile, store_tile, generic);
  } else {
    // state copy only: d <- g, one array each way, whole chunks
    struct Tile {
      u32x4 a[U];
    };
    auto load_tile = [&](const Chunk& ch, Tile& tl) {
      const gvec* gv = reinterpret_cast<const gvec*>(ch.a) + tid;
#pragma unroll
      for (int u = 0; u < U; ++u) tl.a[u] = ld16<GAC_APPLY_NT_LOAD>(gv + u * T);
    };
    auto store_tile = [&](const Chunk& ch, const Tile& tl) {
      gvec* dv = reinterpret_cast<gvec*>(ch.b) + tid;
#pragma unroll
      for (int u = 0; u < U; ++u) st16<GAC_APPLY_NT_STORE>(dv + u * T, tl.a[u]);
    };
    walk_tiles<DT, T, U, Tile>(segs, n_tensors, n_chunks, chunk_elems, work, load_tile, store_tile, generic);
  }
}

// Pass 2 of the buffer-exchange form: the gradient for the optimizer is written over the OLD
// reference state (which nobody needs after this step) and g itself is left alone, because
// the caller hands the g buffers over as the new reference state.  When the step projects
// (or clips): read g, read d, write g' (3 N s bytes); otherwise there is nothing to move.
template <int DT, int T, int U>
__global__ __launch_bounds__(T) void exchange_kernel(const Seg* __restrict__ segs,
                                                            int n_tensors, int64_t n_chunks,
                                                            int chunk_elems,
                                                            const gac_result* __restrict__ res,
                                                            unsigned long long* __restrict__ work) {
  constexpr int N = Elem<DT>::kPerVec;
  if (res->nonfinite || !res->modified) return;
  const float k = static_cast<float>(res->coef_d);
  const float beta = static_cast<float>(res->scale_g);
  const int tid = threadIdx.x;

  typedef PairTile<U> Tile;
  auto load_tile = [&](const Chunk& ch, Tile& tl) {
    const gvec* gv = reinterpret_cast<const gvec*>(ch.a) + tid;
    const gvec* dv = reinterpret_cast<const gvec*>(ch.b) + tid;
#pragma unroll
    for (int u = 0; u < U; ++u) tl.a[u] = ld16<GAC_APPLY_NT_LOAD>(gv + u * T);
#pragma unroll
    for (int u = 0; u < U; ++u) tl.b[u] = ld16<GAC_APPLY_NT_LOAD>(dv + u * T);
  };
  auto store_tile = [&](const Chunk& ch, const Tile& tl) {
    gvec* dv = reinterpret_cast<gvec*>(ch.b) + tid;
#pragma unroll
    for (int u = 0; u < U; ++u)
      st16<GAC_APPLY_NT_STORE>(dv + u * T, project_vec<DT>(tl.a[u], tl.b[u], k, beta));
  };
  auto generic = [&](const Chunk& ch) {
    const gvec* gv = reinterpret_cast<const gvec*>(ch.a);
    gvec* dv = reinterpret_cast<gvec*>(ch.b);
    const int nvec = ch.len / N;
    for (int i = tid; i < nvec; i += T)
      st16<GAC_APPLY_NT_STORE>(dv + i, project_vec<DT>(ld16<GAC_APPLY_NT_LOAD>(gv + i),
                                                       ld16<GAC_APPLY_NT_LOAD>(dv + i), k, beta));
    for (int i = nvec * N + tid; i < ch.len; i += T)
      store_elem<DT>(ch.b, i, fmaf(k, load_elem<DT>(ch.b, i), beta * load_elem<DT>(ch.a, i)));
  };

  walk_tiles<DT, T, U, Tile>(segs, n_tensors, n_chunks, chunk_elems, work, load_tile, store_tile, generic);
}

// Pass 2 of the snapshot form.  Pass 1 has already stored the raw gradient as the next
// reference state, so only a step that projects (or clips) has anything left to do:
// g <- scale_g g + coef_d d_old in place, where d_old is the buffer that stopped being current
// when the finalize step flipped *cur (read g, read d_old, write g: 3 N s bytes).
template <int DT, int T, int U>
__global__ __launch_bounds__(T) void snap_apply_kernel(const Seg* __restrict__ segs,
                                                              int n_tensors, int64_t n_chunks,
                                                              int chunk_elems,
                                                              const gac_result* __restrict__ res,
                                                              unsigned long long* __restrict__ work,
                                                              SnapArgs snap) {
  constexpr int N = Elem<DT>::kPerVec;
  if (res->nonfinite || !res->modified) return;
  const float k = static_cast<float>(res->coef_d);
  const float beta = static_cast<float>(res->scale_g);
  const int64_t old_off = *snap.cur ? 0 : snap.delta;  // the buffer that is no longer current
  const int tid = threadIdx.x;

  typedef PairTile<U> Tile;
  auto load_tile = [&](const Chunk& ch, Tile& tl) {
    const gvec* gv = reinterpret_cast<const gvec*>(ch.a) + tid;
    const gvec* dv = reinterpret_cast<const gvec*>(ch.b + old_off) + tid;
#pragma unroll
    for (int u = 0; u < U; ++u) tl.a[u] = ld16<GAC_APPLY_NT_LOAD>(gv + u * T);
#pragma unroll
    for (int u = 0; u < U; ++u) tl.b[u] = ld16<GAC_APPLY_NT_LOAD>(dv + u * T);
  };
  auto store_tile = [&](const Chunk& ch, const Tile& tl) {
    gvec* gv = reinterpret_cast<gvec*>(const_cast<gchar*>(ch.a)) + tid;
#pragma unroll
    for (int u = 0; u < U; ++u)
      st16<GAC_APPLY_NT_STORE>(gv + u * T, project_vec<DT>(tl.a[u], tl.b[u], k, beta));
  };
  auto generic = [&](const Chunk& ch) {
    gchar* ga = const_cast<gchar*>(ch.a);
    gvec* gv = reinterpret_cast<gvec*>(ga);
    const gvec* dv = reinterpret_cast<const gvec*>(ch.b + old_off);
    const int nvec = ch.len / N;
    for (int i = tid; i < nvec; i += T)
      st16<GAC_APPLY_NT_STORE>(gv + i, project_vec<DT>(ld16<GAC_APPLY_NT_LOAD>(gv + i),
                                                       ld16<GAC_APPLY_NT_LOAD>(dv + i), k, beta));
    for (int i = nvec * N + tid; i < ch.len; i += T)
      store_elem<DT>(ga, i, fmaf(k, load_elem<DT>(ch.b + old_off, i), beta * load_elem<DT>(ch.a, i)));
  };

  walk_tiles<DT, T, U, Tile>(segs, n_tensors, n_chunks, chunk_elems, work, load_tile, store_tile, generic);
}

// ------------------------------------------------------------------ pass 2 fused with AdamW

// One AdamW update of one element (decoupled weight decay) in fp32:
//   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
//   p <- p - [ lr wd p + (lr/(1-b1^t)) m / (sqrt(v)/sqrt(1-b2^t) + eps) ]
// The decay term and the Adam step are added before they are subtracted from p, so p is
// rounded once; with lr wd far below one ulp (1e-8 at the paper's settings) a separate
// p (1 - lr wd) would round to p and lose the decay altogether.
__device__ __forceinline__ void adamw_elem(float g, float& p, float& m, float& v,
                                           const AdamScalars& h) {
  m = fmaf(h.beta1, m, h.one_minus_beta1 * g);
  v = fmaf(h.beta2, v, h.one_minus_beta2 * (g * g));
  const float step = h.step_size * m / (sqrtf(v) * h.inv_sqrt_bc2 + h.eps_adam);
  p = p - fmaf(h.lr_wd, p, step);
}

// Four consecutive gradient elements as stored: 16 bytes of fp32 or 8 bytes of bf16.
template <int DT> struct Quad;
template <> struct Quad<GAC_F32> {
  typedef u32x4 type;
  typedef u32x4_ua stored;  // the same bytes, declared with element alignment only
};
template <> struct Quad<GAC_BF16> {
  typedef u32x2 type;
  typedef u32x2_ua stored;
};

template <int DT>
__device__ __forceinline__ void unpack_quad(typename Quad<DT>::type q, float (&x)[4]) {
  if constexpr (DT == GAC_F32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(q[i]);
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      x[2 * i] = __uint_as_float(q[i] << 16);
      x[2 * i + 1] = __uint_as_float(q[i] & 0xffff0000u);
    }
  }
}

template <int DT>
__device__ __forceinline__ typename Quad<DT>::type pack_quad(const float (&x)[4]) {
  typename Quad<DT>::type q;
  if constexpr (DT == GAC_F32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) q[i] = __float_as_uint(x[i]);
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i) q[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
  }
  return q;
}

// The fused pass works in quads (4 elements): lane l of a workgroup takes quads l, l+T, ...
// so that every load and store instruction of a wave covers one contiguous range, both for
// the 2-byte gradient / state (8 bytes per lane) and for the 4-byte optimizer state (16 bytes
// per lane).

// The arithmetic of one quad: g' = scale_g g + coef_d d where the step projects and/or clips,
// then AdamW on p, m, v (updated in place); pnew receives the new parameters.
template <int DT>
__device__ __forceinline__ void adamw_quad(typename Quad<DT>::type a, typename Quad<DT>::type b,
                                           u32x4& P, u32x4& M, u32x4& V, float (&pnew)[4],
                                           bool project, float k, float beta, const AdamScalars& h) {
  float x[4];
  unpack_quad<DT>(a, x);
  if (project) {
    float y[4];
    unpack_quad<DT>(b, y);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = fmaf(k, y[e], beta * x[e]);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float p = __uint_as_float(P[e]), m = __uint_as_float(M[e]), v = __uint_as_float(V[e]);
    adamw_elem(x[e], p, m, v, h);
    P[e] = __float_as_uint(p);
    M[e] = __float_as_uint(m);
    V[e] = __float_as_uint(v);
    pnew[e] = p;
  }
}

// One quad from memory to memory (units that are not a whole tile).
template <int DT, int NTL>
__device__ __forceinline__ void adamw_single_quad(const gchar* ga, gchar* gb, gfloat* pp, gfloat* pm,
                                                  gfloat* pv, gchar* pl, int j, bool project,
                                                  bool skip, float k, float beta,
                                                  const AdamScalars& h) {
  typedef typename Quad<DT>::type quad_t;
  typedef GAC_GLOBAL typename Quad<DT>::stored gquad;
  const gquad* gq = reinterpret_cast<const gquad*>(ga) + j;
  gquad* dq = reinterpret_cast<gquad*>(gb) + j;
  quad_t a, b = {};
  if constexpr (NTL) {
    a = __builtin_nontemporal_load(gq);
  } else {
    a = *gq;
  }
  if (skip) {  // violation: only the reference state moves, the optimizer is untouched
    __builtin_nontemporal_store(a, dq);
    return;
  }
  if (project) {
    if constexpr (NTL) {
      b = __builtin_nontemporal_load(dq);
    } else {
      b = *dq;
    }
  }
  gvec* vp = reinterpret_cast<gvec*>(pp) + j;
  gvec* vm = reinterpret_cast<gvec*>(pm) + j;
  gvec* vv = reinterpret_cast<gvec*>(pv) + j;
  u32x4 P = ld16<NTL>(vp), M = ld16<NTL>(vm), V = ld16<NTL>(vv);
  float pnew[4];
  adamw_quad<DT>(a, b, P, M, V, pnew, project, k, beta, h);
  st16<1>(vp, P);
  st16<1>(vm, M);
  st16<1>(vv, V);
  __builtin_nontemporal_store(a, dq);
  if (pl != nullptr) __builtin_nontemporal_store(pack_quad<DT>(pnew), reinterpret_cast<gquad*>(pl) + j);
}

// Pass 2 with the optimizer fused in.  The traversal is that of the other pass-2 kernels
// (walk_tiles): a tile is T x Q quads of each of the five arrays (a quarter of a default bf16
// chunk, half of an fp32 one), and the next tile's loads are issued before the current tile
// is computed and stored, so that reads stay in flight while the workgroup stores.

// One tile of the fused pass in registers: Q quads per lane of g, d, p, m and v.
template <int DT, int Q>
struct AdamTile {
  typename Quad<DT>::type a[Q], b[Q];
  u32x4 P[Q], M[Q], V[Q];
};

template <int DT, int T>
__global__ __launch_bounds__(T) void apply_adamw_kernel(
    const Seg* __restrict__ segs, const AdamSeg* __restrict__ adam, int n_tensors,
    int64_t n_chunks, int chunk_elems, const gac_result* __restrict__ res,
    unsigned long long* __restrict__ work, AdamScalars h) {
  constexpr int Q = GAC_ADAMW_QUADS;             // quads per lane and array in one tile
  constexpr int N = Elem<DT>::kPerVec;
  constexpr int U = Q * 4 / N;                   // the tile's length in 16-byte vectors of g per lane
  constexpr int kTileElems = T * Q * 4;
  constexpr int kChunkElems = kDefaultChunkBytes / Elem<DT>::kSize;
  constexpr int SPLIT = kChunkElems / kTileElems;  // tiles in a chunk of the default size
  static_assert(U >= 1 && U * N == Q * 4, "a tile is a whole number of gradient vectors per lane");
  static_assert(SPLIT >= 1 && SPLIT * kTileElems == kChunkElems, "tiles divide the default chunk");
  typedef GAC_GLOBAL typename Quad<DT>::stored gquad;
  if (res->nonfinite) return;
  const bool project = res->modified != 0;  // projected and/or clipped
  const bool skip = res->regime == GAC_SKIP;
  const float k = static_cast<float>(res->coef_d);
  const float beta = static_cast<float>(res->scale_g);
  const int tid = threadIdx.x;

  typedef AdamTile<DT, Q> Tile;
  auto load_tile = [&](const Chunk& ch, Tile& tl) {
    const gquad* gq = reinterpret_cast<const gquad*>(ch.a) + tid;
#pragma unroll
    for (int q = 0; q < Q; ++q) tl.a[q] = __builtin_nontemporal_load(gq + q * T);
    if (skip) return;  // violation: only the reference state moves
    if (project) {
      const gquad* dq = reinterpret_cast<const gquad*>(ch.b) + tid;
#pragma unroll
      for (int q = 0; q < Q; ++q) tl.b[q] = __builtin_nontemporal_load(dq + q * T);
    }
    const AdamSeg as = adam[ch.tensor];
    const gvec* vp = reinterpret_cast<const gvec*>((const gfloat*)(as.p) + ch.elem_off) + tid;
    const gvec* vm = reinterpret_cast<const gvec*>((const gfloat*)(as.m) + ch.elem_off) + tid;
    const gvec* vv = reinterpret_cast<const gvec*>((const gfloat*)(as.v) + ch.elem_off) + tid;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      tl.P[q] = ld16<GAC_ADAMW_NT_LOAD>(vp + q * T);
      tl.M[q] = ld16<GAC_ADAMW_NT_LOAD>(vm + q * T);
      tl.V[q] = ld16<GAC_ADAMW_NT_LOAD>(vv + q * T);
    }
  };
  auto store_tile = [&](const Chunk& ch, const Tile& tl) {
    gquad* dq = reinterpret_cast<gquad*>(ch.b) + tid;
    if (skip) {
#pragma unroll
      for (int q = 0; q < Q; ++q) __builtin_nontemporal_store(tl.a[q], dq + q * T);
      return;
    }
    const AdamSeg as = adam[ch.tensor];
    gvec* vp = reinterpret_cast<gvec*>((gfloat*)(as.p) + ch.elem_off) + tid;
    gvec* vm = reinterpret_cast<gvec*>((gfloat*)(as.m) + ch.elem_off) + tid;
    gvec* vv = reinterpret_cast<gvec*>((gfloat*)(as.v) + ch.elem_off) + tid;
    gquad* lq = as.p_lowp ? reinterpret_cast<gquad*>((gchar*)(as.p_lowp) + ch.elem_off * Elem<DT>::kSize) + tid : nullptr;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      u32x4 P = tl.P[q], M = tl.M[q], V = tl.V[q];
      float pnew[4];
      adamw_quad<DT>(tl.a[q], tl.b[q], P, M, V, pnew, project, k, beta, h);
      st16<1>(vp + q * T, P);
      st16<1>(vm + q * T, M);
      st16<1>(vv + q * T, V);
      __builtin_nontemporal_store(tl.a[q], dq + q * T);
      if (lq != nullptr) __builtin_nontemporal_store(pack_quad<DT>(pnew), lq + q * T);
    }
  };
  // a unit that is not a whole tile: single quads per lane, then single elements
  auto generic = [&](const Chunk& ch) {
    const AdamSeg as = adam[ch.tensor];
    gfloat* pp = (gfloat*)(as.p) + ch.elem_off;
    gfloat* pm = (gfloat*)(as.m) + ch.elem_off;
    gfloat* pv = (gfloat*)(as.v) + ch.elem_off;
    gchar* pl = as.p_lowp ? (gchar*)(as.p_lowp) + ch.elem_off * Elem<DT>::kSize : nullptr;
    const int nquad = ch.len / 4;
    for (int j = tid; j < nquad; j += T)
      adamw_single_quad<DT, GAC_ADAMW_NT_LOAD>(ch.a, ch.b, pp, pm, pv, pl, j, project, skip, k, beta, h);
    for (int i = nquad * 4 + tid; i < ch.len; i += T) {
      if (!skip) {
        float g = load_elem<DT>(ch.a, i);
        if (project) g = fmaf(k, load_elem<DT>(ch.b, i), beta * g);
        float p = pp[i], m = pm[i], v = pv[i];
        adamw_elem(g, p, m, v, h);
        pp[i] = p;
        pm[i] = m;
        pv[i] = v;
        if (pl != nullptr) store_elem<DT>(pl, i, p);
      }
      copy_elem<DT>(ch.a, ch.b, i);
    }
  };
  walk_tiles<DT, T, U, Tile, SPLIT>(segs, n_tensors, n_chunks, chunk_elems, work, load_tile, store_tile, generic);
}
// ------------------------------------------------------------------ alignment statistics

// Table 3 of the paper: the 0.9-quantile and the maximum of |c_t| and the share of steps
// with |c_t| <= c_low, over recorded steps first_step .. last_step.  One workgroup: the
// |c_t| go to LDS (missing and non-finite entries as +inf, which sort to the end), a bitonic
// sort orders them, thread 0 interpolates the quantile at position (m-1) * 0.9.
__global__ __launch_bounds__(1024) void diag_kernel(const double* __restrict__ hist_c,
                                                    const int32_t* __restrict__ hist_regime,
                                                    int hist_cap, int64_t first_step,
                                                    int64_t last_step, double c_low,
                                                    gac_diag* __restrict__ out,
                                                    gac_diag* __restrict__ host_out) {
  __shared__ double a[kMaxHistory];
  __shared__ int counts[5];  // safe, projected, skipped, non-finite, |c| <= c_low
  const int tid = threadIdx.x;
  if (tid < 5) counts[tid] = 0;
  __syncthreads();
  const int64_t n_steps = last_step >= first_step ? last_step - first_step + 1 : 0;
  const double inf = __longlong_as_double(0x7ff0000000000000LL);
  for (int i = tid; i < kMaxHistory; i += 1024) {
    double v = inf;
    if (i < n_steps) {
      const int slot = static_cast<int>((first_step + i - 1) % hist_cap);
      const int regime = hist_regime[slot];
      if (regime < 0) {
        atomicAdd(&counts[3], 1);
      } else {
        v = fabs(hist_c[slot]);
        atomicAdd(&counts[regime], 1);
        if (v <= c_low) atomicAdd(&counts[4], 1);
      }
    }
    a[i] = v;
  }
  __syncthreads();
  for (int size = 2; size <= kMaxHistory; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < kMaxHistory / 2; i += 1024) {
        const int lo = 2 * i - (i & (stride - 1));  // index with bit `stride` clear
        const int hi = lo + stride;
        const bool ascending = (lo & size) == 0;
        const double x = a[lo], y = a[hi];
        if ((x > y) == ascending) {
          a[lo] = y;
          a[hi] = x;
        }
      }
      __syncthreads();
    }
  }
  if (tid != 0) return;
  gac_diag d;
  d.first_step = first_step;
  d.last_step = last_step;
  d.n_nonfinite = counts[3];
  d.regime_count[0] = counts[0];
  d.regime_count[1] = counts[1];
  d.regime_count[2] = counts[2];
  const int m = counts[0] + counts[1] + counts[2];
  d.n_values = m;
  d.q90_abs_c = 0.0;
  d.max_abs_c = 0.0;
  d.frac_le_c_low = 0.0;
  if (m > 0) {
    const double pos = (static_cast<double>(m) - 1.0) * 0.9;
    const int lo = static_cast<int>(floor(pos));
    const int hi = lo + 1 < m ? lo + 1 : m - 1;
    d.q90_abs_c = a[lo] + (a[hi] - a[lo]) * (pos - static_cast<double>(lo));
    d.max_abs_c = a[m - 1];
    d.frac_le_c_low = static_cast<double>(counts[4]) / static_cast<double>(m);
  }
  *out = d;
  if (host_out != nullptr) *host_out = d;
}

// Section 4.2 rule applied to the recorded c_t under other threshold pairs: one workgroup
// per pair, counts combined in LDS, three integers per pair written to host-mapped memory.
__global__ __launch_bounds__(kThreads) void sweep_kernel(const double* __restrict__ hist_c,
                                                         const int32_t* __restrict__ hist_regime,
                                                         int hist_cap, int64_t first_step,
                                                         int64_t last_step, SweepPairs pairs,
                                                         int32_t* __restrict__ host_counts) {
  __shared__ int counts[3];
  const int tid = threadIdx.x;
  if (tid < 3) counts[tid] = 0;
  __syncthreads();
  const double c_low = pairs.c_low[blockIdx.x], c_high = pairs.c_high[blockIdx.x];
  const int64_t n_steps = last_step >= first_step ? last_step - first_step + 1 : 0;
  int mine[3] = {0, 0, 0};
  for (int64_t i = tid; i < n_steps; i += kThreads) {
    const int slot = static_cast<int>((first_step + i - 1) % hist_cap);
    if (hist_regime[slot] < 0) continue;  // non-finite step: no cosine
    const double mag = fabs(hist_c[slot]);
    const int regime = mag <= c_low ? GAC_SAFE : (mag >= c_high ? GAC_SKIP : GAC_PROJECT);
    mine[0] += regime == GAC_SAFE;
    mine[1] += regime == GAC_PROJECT;
    mine[2] += regime == GAC_SKIP;
  }
  for (int r = 0; r < 3; ++r)
    if (mine[r]) atomicAdd(&counts[r], mine[r]);
  __syncthreads();
  if (tid < 3) host_counts[3 * blockIdx.x + tid] = counts[tid];
}

// ------------------------------------------------------------------ state maintenance

// op kStateZero: b <- 0;  op kStateCopy: b <- a.   (init / reset / export / import)
template <int DT>
__global__ __launch_bounds__(kThreads) void state_kernel(const Seg* __restrict__ segs,
                                                         int64_t n_chunks, int chunk_elems,
                                                         int op) {
  constexpr int N = Elem<DT>::kPerVec;
  const int tid = threadIdx.x;
  int t = 0;
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const Chunk ch = locate<false>(segs, t, c, chunk_elems, Elem<DT>::kSize);
    const gvec* src = reinterpret_cast<const gvec*>(ch.a);
    gvec* dst = reinterpret_cast<gvec*>(ch.b);
    const int nvec = ch.len / N;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int i = tid; i < nvec; i += kThreads) dst[i] = (op == kStateZero) ? zero : src[i];
    const int first_scalar = nvec * N;
    for (int i = first_scalar + tid; i < ch.len; i += kThreads) {
      if (op == kStateZero) {
        if constexpr (DT == GAC_F32) {
          reinterpret_cast<gu32*>(ch.b)[i] = 0u;
        } else {
          reinterpret_cast<gu16*>(ch.b)[i] = 0u;
        }
      } else {
        copy_elem<DT>(ch.a, ch.b, i);
      }
    }
  }
}

}  // namespace

// Workgroups of the fused AdamW kernel that fit on one CU at the same time.
int adamw_blocks_per_cu(int dtype) {
  int n = 0;
  hipError_t e = dtype == GAC_F32
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &n, apply_adamw_kernel<GAC_F32, GAC_ADAMW_THREADS>, GAC_ADAMW_THREADS, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &n, apply_adamw_kernel<GAC_BF16, GAC_ADAMW_THREADS>, GAC_ADAMW_THREADS, 0);
  return (e == hipSuccess && n > 0) ? n : 1;
}

// ------------------------------------------------------------------ launchers

namespace {
FinalArgs final_args(const double* sums_in, double* sums_out, gac_result* dev_result,
                     gac_result* host_result, const DecideParams& p, int mode) {
  FinalArgs f;
  f.sums_in = sums_in;
  f.sums_out = sums_out;
  f.res = dev_result;
  f.host_res = host_result;
  f.p = p;
  f.mode = mode;
  return f;
}
}  // namespace

hipError_t launch_reduce(int dtype, const Seg* dev_segs, int64_t n_chunks, int chunk_elems,
                         double* dev_partials, unsigned int* dev_ticket, int grid, double* sums_out,
                         gac_result* dev_result, gac_result* host_result, DecideParams p, int mode,
                         hipStream_t stream) {
  // the combine of the folded finalize step must be the one of the stand-alone kernel, bit for bit
  static_assert(GAC_REDUCE_THREADS == kThreads, "the fixed-order combine assumes kThreads lanes");
  const FinalArgs f = final_args(nullptr, sums_out, dev_result, host_result, p, mode | 1);
  constexpr int T = GAC_REDUCE_THREADS, U = GAC_REDUCE_UNROLL;
  if (dtype == GAC_F32) {
    reduce_kernel<GAC_F32, T, U><<<grid, T, 0, stream>>>(dev_segs, n_chunks, chunk_elems, dev_partials, dev_ticket, f);
  } else {
    reduce_kernel<GAC_BF16, T, U><<<grid, T, 0, stream>>>(dev_segs, n_chunks, chunk_elems, dev_partials, dev_ticket, f);
  }
  return hipGetLastError();
}

int64_t snap_group_count(int64_t n_chunks) { return (n_chunks + kSnapGroup - 1) / kSnapGroup; }

hipError_t launch_snap_reduce(int dtype, const Seg* dev_segs, int64_t n_chunks, int chunk_elems,
                              const SnapBuffers& b, int grid, double* sums_out, gac_result* dev_result,
                              gac_result* host_result, DecideParams p, int mode, int64_t snap_delta,
                              hipStream_t stream) {
  const FinalArgs f = final_args(nullptr, sums_out, dev_result, host_result, p, mode | 1);
  const SnapArgs sn = {p.cur, snap_delta};
  const SnapWork w = {b.draw, b.chunk_sums, b.group_sums, b.ticket};
  if (dtype == GAC_F32) {
    snap_reduce_kernel<GAC_F32><<<grid, kSnapThreads, 0, stream>>>(dev_segs, n_chunks, chunk_elems, w, sn);
  } else {
    snap_reduce_kernel<GAC_BF16><<<grid, kSnapThreads, 0, stream>>>(dev_segs, n_chunks, chunk_elems, w, sn);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t n_groups = snap_group_count(n_chunks);
  const int combine_grid = static_cast<int>(n_groups < 1 ? 1 : (n_groups > 1024 ? 1024 : n_groups));
  snap_combine_kernel<<<combine_grid, kThreads, 0, stream>>>(n_chunks, w, f);
  return hipGetLastError();
}

hipError_t launch_finalize(const double* sums_in, double* sums_out, gac_result* dev_result,
                           gac_result* host_result, DecideParams p, hipStream_t stream) {
  finalize_kernel<<<1, kThreads, 0, stream>>>(
      nullptr, 0, final_args(sums_in, sums_out, dev_result, host_result, p, /*mode=*/2));
  return hipGetLastError();
}

hipError_t launch_apply(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                        int chunk_elems, const gac_result* dev_result, unsigned long long* dev_work,
                        int grid, hipStream_t stream) {
  if (dtype == GAC_F32) {
    apply_kernel<GAC_F32, GAC_APPLY_THREADS, GAC_APPLY_UNROLL, false><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, dev_result, dev_work, 0.0f, 1.0f);
  } else {
    apply_kernel<GAC_BF16, GAC_APPLY_THREADS, GAC_APPLY_UNROLL, false><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, dev_result, dev_work, 0.0f, 1.0f);
  }
  return hipGetLastError();
}

hipError_t launch_apply_probe(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                              int chunk_elems, unsigned long long* dev_work, int grid,
                              hipStream_t stream) {
  if (dtype == GAC_F32) {
    apply_kernel<GAC_F32, GAC_APPLY_THREADS, GAC_APPLY_UNROLL, true><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, nullptr, dev_work, 0.0f, 1.0f);
  } else {
    apply_kernel<GAC_BF16, GAC_APPLY_THREADS, GAC_APPLY_UNROLL, true><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, nullptr, dev_work, 0.0f, 1.0f);
  }
  return hipGetLastError();
}

hipError_t launch_exchange(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                           int chunk_elems, const gac_result* dev_result,
                           unsigned long long* dev_work, int grid, hipStream_t stream) {
  if (dtype == GAC_F32) {
    exchange_kernel<GAC_F32, GAC_APPLY_THREADS, GAC_APPLY_UNROLL><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, dev_result, dev_work);
  } else {
    exchange_kernel<GAC_BF16, GAC_APPLY_THREADS, GAC_APPLY_UNROLL><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, dev_result, dev_work);
  }
  return hipGetLastError();
}

hipError_t launch_snap_apply(int dtype, const Seg* dev_segs, int n_tensors, int64_t n_chunks,
                             int chunk_elems, const gac_result* dev_result,
                             unsigned long long* dev_work, int32_t* dev_cur, int64_t snap_delta,
                             int grid, hipStream_t stream) {
  const SnapArgs sn = {dev_cur, snap_delta};
  if (dtype == GAC_F32) {
    snap_apply_kernel<GAC_F32, GAC_APPLY_THREADS, GAC_APPLY_UNROLL><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, dev_result, dev_work, sn);
  } else {
    snap_apply_kernel<GAC_BF16, GAC_APPLY_THREADS, GAC_APPLY_UNROLL><<<grid, GAC_APPLY_THREADS, 0, stream>>>(
        dev_segs, n_tensors, n_chunks, chunk_elems, dev_result, dev_work, sn);
  }
  return hipGetLastError();
}

hipError_t launch_apply_adamw(int dtype, const Seg* dev_segs, const AdamSeg* dev_adam,
                              int n_tensors, int64_t n_chunks, int chunk_elems,
                              const gac_result* dev_result, unsigned long long* dev_work,
                              AdamScalars h, int grid, hipStream_t stream) {
  if (dtype == GAC_F32) {
    apply_adamw_kernel<GAC_F32, GAC_ADAMW_THREADS><<<grid, GAC_ADAMW_THREADS, 0, stream>>>(
        dev_segs, dev_adam, n_tensors, n_chunks, chunk_elems, dev_result, dev_work, h);
  } else {
    apply_adamw_kernel<GAC_BF16, GAC_ADAMW_THREADS><<<grid, GAC_ADAMW_THREADS, 0, stream>>>(
        dev_segs, dev_adam, n_tensors, n_chunks, chunk_elems, dev_result, dev_work, h);
  }
  return hipGetLastError();
}

hipError_t launch_diag(const double* hist_c, const int32_t* hist_regime, int hist_cap,
                       int64_t first_step, int64_t last_step, double c_low, gac_diag* dev_out,
                       gac_diag* host_out, hipStream_t stream) {
  diag_kernel<<<1, 1024, 0, stream>>>(hist_c, hist_regime, hist_cap, first_step, last_step, c_low,
                                      dev_out, host_out);
  return hipGetLastError();
}

hipError_t launch_sweep(const double* hist_c, const int32_t* hist_regime, int hist_cap,
                        int64_t first_step, int64_t last_step, const SweepPairs& pairs,
                        int n_pairs, int32_t* host_counts, hipStream_t stream) {
  sweep_kernel<<<n_pairs, kThreads, 0, stream>>>(hist_c, hist_regime, hist_cap, first_step,
                                                 last_step, pairs, host_counts);
  return hipGetLastError();
}

namespace {
__global__ void set_step_kernel(int64_t* dev_step, int64_t value) { *dev_step = value; }
__global__ void set_word_kernel(uint32_t* dev_word, uint32_t value) { *dev_word = value; }

// Writes `count` entries of the tensor table from the kernel's own arguments (so the table
// reaches the device without a copy command and without staging memory) and, with the first
// batch, clears the ticket counter of the reduction.
__global__ __launch_bounds__(kSegBatch) void fill_segs_kernel(Seg* __restrict__ table, SegBatch b,
                                                              unsigned int* __restrict__ ticket) {
  const int i = threadIdx.x;
  if (i < b.count) table[b.first + i] = b.e[i];
  if (ticket != nullptr && i == 0) *ticket = 0u;
}
}  // namespace

hipError_t launch_set_step(int64_t* dev_step, int64_t value, hipStream_t stream) {
  set_step_kernel<<<1, 1, 0, stream>>>(dev_step, value);
  return hipGetLastError();
}

hipError_t launch_set_word(uint32_t* dev_word, uint32_t value, hipStream_t stream) {
  set_word_kernel<<<1, 1, 0, stream>>>(dev_word, value);
  return hipGetLastError();
}

hipError_t launch_fill_segs(Seg* dev_table, const SegBatch& batch, unsigned int* ticket_to_clear,
                            hipStream_t stream) {
  fill_segs_kernel<<<1, kSegBatch, 0, stream>>>(dev_table, batch, ticket_to_clear);
  return hipGetLastError();
}

// ------------------------------------------------------------------ static scratch

// Device memory of the entry point that allocates nothing (gac_step_static): the tensor
// table, the per-workgroup partial sums, the ticket counter, the three sums and the result
// record that the context-based entry points keep in memory from hipMalloc.  Every GPU the
// library runs on holds its own copy of this array, at its own address, until the process
// ends.  In host code the name is only a handle for hipGetSymbolAddress: the address that
// kernels can use is looked up once per device and kept in g_scratch_ptr.
namespace {
constexpr size_t kScratchTicketOff = 0;
constexpr size_t kScratchWorkOff = 8;
constexpr size_t kScratchSumsOff = 64;
constexpr size_t kScratchResultOff = 128;
constexpr size_t kScratchPartialsOff = 256;
constexpr size_t kScratchSegsOff = kScratchPartialsOff + sizeof(double) * 3 * kStaticMaxGrid;
constexpr size_t kScratchBytes =
    (kScratchSegsOff + sizeof(Seg) * (kStaticMaxTensors + 1) + 255) / 256 * 256;
static_assert(sizeof(gac_result) <= kScratchPartialsOff - kScratchResultOff, "result slot too small");
static_assert(kScratchSegsOff % 32 == 0, "tensor table alignment");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

size_t static_scratch_bytes() { return kScratchBytes; }

hipError_t static_scratch(int device, StaticScratch* out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
      // `device` is the current device here: the symbol resolves to this GPU's copy
      void* ptr = nullptr;
      const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (ptr == nullptr) return hipErrorInvalidSymbol;
      g_scratch_ptr[device] = ptr;
    }
    base = g_scratch_ptr[device];
  }
  unsigned char* b = static_cast<unsigned char*>(base);
  out->ticket = reinterpret_cast<unsigned int*>(b + kScratchTicketOff);
  out->work = reinterpret_cast<unsigned long long*>(b + kScratchWorkOff);
  out->sums = reinterpret_cast<double*>(b + kScratchSumsOff);
  out->result = reinterpret_cast<gac_result*>(b + kScratchResultOff);
  out->partials = reinterpret_cast<double*>(b + kScratchPartialsOff);
  out->segs = reinterpret_cast<Seg*>(b + kScratchSegsOff);
  return hipSuccess;
}

hipError_t launch_state_op(int dtype, int op, const Seg* dev_segs, int64_t n_chunks,
                           int chunk_elems, int grid, hipStream_t stream) {
  if (dtype == GAC_F32) {
    state_kernel<GAC_F32><<<grid, kThreads, 0, stream>>>(dev_segs, n_chunks, chunk_elems, op);
  } else {
    state_kernel<GAC_BF16><<<grid, kThreads, 0, stream>>>(dev_segs, n_chunks, chunk_elems, op);
  }
  return hipGetLastError();
}

}  // namespace gac
