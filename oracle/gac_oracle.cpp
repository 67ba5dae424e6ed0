// GAC oracle: a plain, slow, single-threaded CPU statement of what one Gradient
// Alignment Control update computes.  TEST INFRASTRUCTURE ONLY: it exists so
// that the GPU library can be checked against something written straight from
// the paper.  It shares no code, header, table or helper with the GPU library,
// and no product code path may call it.
//
// Everything is fp64, sums run left to right over the tensor list in order,
// nothing is blocked, fused or reordered.
//
// What it follows (paper: "GAC: Stabilizing Asynchronous RL Training for LLMs
// via Gradient Alignment Control", arXiv 2603.01501):
//   * statistics and cosine with epsilon ........ Appendix A.1 (three dot
//     products; c = <g,d> / (sqrt(|g|^2 |d|^2) + eps)), Eq. 1
//   * regimes (safe / projection / violation) ... Section 4.2, Algorithm 1
//   * directional decomposition and rescale ..... Eq. 2, Eq. 3, Eq. 4
//   * rank-one form with alpha = c_low/|c| ...... Appendix A.2
//   * reference state = previous raw gradient,
//     initialised to zero ....................... Algorithm 1, Appendix A.2
//   * AdamW hyper-parameters .................... Table 2 (the update rule
//     itself is the textbook decoupled-weight-decay Adam)
//   * gradient clipping ......................... Table 2 lists it as on, without
//     order or threshold: read as global-norm clipping of the gradient GAC hands
//     to the optimizer, scale = min(1, max_norm / (norm + 1e-6)) (the convention
//     of the framework the paper builds on)
//   * alignment statistics ...................... Table 3: q0.9(|c_t|), max |c_t|,
//     Pr(|c_t| <= 0.05) over the updates after a burn-in
//
// Readings taken where the paper is silent are listed next to each function.
// Parity status: every function here is pinned by tests that do not go through
// this file's own arithmetic (closed forms, hand-worked length-8 cases, numpy
// dot products, torch.optim.AdamW in fp64); nothing is "parity unpinned"
// except the non-finite convention of gac_oracle_decide, which the paper does
// not define.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// Storage dtypes of gradient / state elements.
constexpr int kF32 = 0;
constexpr int kBF16 = 1;

// bfloat16 is the upper 16 bits of an IEEE binary32; widening is exact.
inline double bf16_to_f64(uint16_t h) {
  uint32_t w = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &w, sizeof f);
  return static_cast<double>(f);
}

inline double load(const void* p, int64_t i, int dtype) {
  if (dtype == kBF16) return bf16_to_f64(static_cast<const uint16_t*>(p)[i]);
  return static_cast<double>(static_cast<const float*>(p)[i]);
}

inline int64_t elem_size(int dtype) { return dtype == kBF16 ? 2 : 4; }

}  // namespace

extern "C" {

// Regime codes (Section 4.2).
enum { ORACLE_SAFE = 0, ORACLE_PROJECT = 1, ORACLE_SKIP = 2 };

struct gac_oracle_decision {
  double c;        // cosine with epsilon (Appendix A.1)
  double alpha;    // c_low / |c| in the projection regime, else 1
  int32_t regime;  // ORACLE_*
  int32_t nonfinite;
};

// Appendix A.1: the three inner products over the flattened concatenation of
// all tensors, here summed tensor by tensor, element by element, in fp64.
//   out[0] = <g,d>   out[1] = <g,g>   out[2] = <d,d>
void gac_oracle_sums(int32_t n_tensors, const void* const* g,
                     const void* const* d, const int64_t* numel, int32_t dtype,
                     double out[3]) {
  double s_gd = 0.0, s_gg = 0.0, s_dd = 0.0;
  for (int32_t j = 0; j < n_tensors; ++j) {
    for (int64_t i = 0; i < numel[j]; ++i) {
      const double gi = load(g[j], i, dtype);
      const double di = load(d[j], i, dtype);
      s_gd += gi * di;
      s_gg += gi * gi;
      s_dd += di * di;
    }
  }
  out[0] = s_gd;
  out[1] = s_gg;
  out[2] = s_dd;
}

// Cosine (Appendix A.1: epsilon is added to the square root, not under it) and
// the three-way branch of Algorithm 1, in the order the algorithm tests them:
// first |c| <= c_low (safe), then |c| >= c_high (violation), else projection
// with alpha = c_low / |c|.
//
// Reading (paper silent): if any of the sums is not finite the step is
// reported as nonfinite with regime SKIP and alpha = 1.
void gac_oracle_decide(const double sums[3], double c_low, double c_high,
                       double eps, gac_oracle_decision* out) {
  const double s_gd = sums[0], s_gg = sums[1], s_dd = sums[2];
  out->nonfinite = 0;
  out->alpha = 1.0;
  if (!std::isfinite(s_gd) || !std::isfinite(s_gg) || !std::isfinite(s_dd)) {
    out->nonfinite = 1;
    out->c = std::nan("");
    out->regime = ORACLE_SKIP;
    return;
  }
  const double c = s_gd / (std::sqrt(s_gg * s_dd) + eps);
  out->c = c;
  const double a = std::fabs(c);
  if (a <= c_low) {
    out->regime = ORACLE_SAFE;
  } else if (a >= c_high) {
    out->regime = ORACLE_SKIP;
  } else {
    out->regime = ORACLE_PROJECT;
    out->alpha = c_low / a;
  }
}

// Eq. 2 - Eq. 4 / Algorithm 1 written out literally for one tensor of the
// list: u = d / |d|, g_par = <g,u> u, g_perp = g - g_par,
// g' = alpha g_par + beta g_perp.  <g,u> and |d| are global (whole list)
// quantities, so they come from the sums:  <g,u> = S_gd / sqrt(S_dd).
// No epsilon appears here (the paper puts it only in the cosine).
void gac_oracle_project_decomposed(const void* g, const void* d, int64_t n,
                                   int32_t dtype, const double sums[3],
                                   double alpha, double beta, double* g_out) {
  const double norm_d = std::sqrt(sums[2]);
  const double g_dot_u = sums[0] / norm_d;
  for (int64_t i = 0; i < n; ++i) {
    const double gi = load(g, i, dtype);
    const double ui = load(d, i, dtype) / norm_d;
    const double g_par = g_dot_u * ui;
    const double g_perp = gi - g_par;
    g_out[i] = alpha * g_par + beta * g_perp;
  }
}

// The same map in the rank-one form of Section 4.1 / Appendix A.2:
// g' = beta g + (alpha - beta) <g,u> u, with <g,u> u = (S_gd / S_dd) d.
void gac_oracle_project_rank_one(const void* g, const void* d, int64_t n,
                                 int32_t dtype, const double sums[3],
                                 double alpha, double beta, double* g_out) {
  const double k = (alpha - beta) * (sums[0] / sums[2]);
  for (int64_t i = 0; i < n; ++i) {
    g_out[i] = beta * load(g, i, dtype) + k * load(d, i, dtype);
  }
}

// Safe and violation regimes leave the gradient as it is (Algorithm 1 uses the
// raw gradient in the safe branch and no gradient at all in the skip branch).
void gac_oracle_passthrough(const void* g, int64_t n, int32_t dtype,
                            double* g_out) {
  for (int64_t i = 0; i < n; ++i) g_out[i] = load(g, i, dtype);
}

// Reference-state update: the next step compares against the RAW gradient of
// this step (Algorithm 1 uses the un-primed g_{t-1}; Appendix A.1 computes the
// cosine on raw gradients before any GAC intervention), in every regime.  The
// state has the gradient's dtype, so this is a bit copy.
void gac_oracle_snapshot(const void* g, void* d, int64_t n, int32_t dtype) {
  std::memcpy(d, g, static_cast<size_t>(n * elem_size(dtype)));
}

// One whole update over a tensor list.  g_out[j] (fp64, numel[j] elements)
// receives the gradient the optimizer should see; d[j] is overwritten with the
// raw g[j] afterwards.  Reading (paper silent): a nonfinite step leaves the
// state untouched.  Returns the regime.
int32_t gac_oracle_step(int32_t n_tensors, const void* const* g,
                        void* const* d, const int64_t* numel, int32_t dtype,
                        double c_low, double c_high, double eps,
                        double* const* g_out, double sums_out[3],
                        gac_oracle_decision* dec_out) {
  double sums[3];
  gac_oracle_sums(n_tensors, g, d, numel, dtype, sums);
  gac_oracle_decision dec;
  gac_oracle_decide(sums, c_low, c_high, eps, &dec);
  for (int32_t j = 0; j < n_tensors; ++j) {
    if (g_out != nullptr && g_out[j] != nullptr) {
      if (dec.regime == ORACLE_PROJECT) {
        gac_oracle_project_decomposed(g[j], d[j], numel[j], dtype, sums,
                                      dec.alpha, 1.0, g_out[j]);
      } else {
        gac_oracle_passthrough(g[j], numel[j], dtype, g_out[j]);
      }
    }
  }
  if (!dec.nonfinite) {
    for (int32_t j = 0; j < n_tensors; ++j)
      gac_oracle_snapshot(g[j], d[j], numel[j], dtype);
  }
  if (sums_out != nullptr) std::memcpy(sums_out, sums, sizeof sums);
  if (dec_out != nullptr) *dec_out = dec;
  return dec.regime;
}

// Textbook AdamW (Adam with decoupled weight decay), one step on one tensor,
// all in fp64, hyper-parameters as in Table 2.  Operation order (the GPU
// kernel follows the same order):
//   m <- b1 m + (1-b1) g
//   v <- b2 v + (1-b2) g^2
//   p <- p - lr wd p
//   p <- p - lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
// g is the (already projected) gradient in fp64: it is NOT rounded to the
// storage dtype in between.  Descent form: g is the gradient of the loss.
// m, v, p are read as fp32 and the new values are returned in fp64.
void gac_oracle_adamw(const double* g, const float* p, const float* m,
                      const float* v, int64_t n, double lr, double beta1,
                      double beta2, double eps_adam, double weight_decay,
                      int64_t t, double* p_out, double* m_out, double* v_out) {
  const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(t));
  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(t));
  for (int64_t i = 0; i < n; ++i) {
    const double gi = g[i];
    const double mi = beta1 * static_cast<double>(m[i]) + (1.0 - beta1) * gi;
    const double vi = beta2 * static_cast<double>(v[i]) + (1.0 - beta2) * gi * gi;
    double pi = static_cast<double>(p[i]);
    pi = pi - lr * weight_decay * pi;
    pi = pi - lr * (mi / bc1) / (std::sqrt(vi / bc2) + eps_adam);
    m_out[i] = mi;
    v_out[i] = vi;
    p_out[i] = pi;
  }
}

// Global-norm clipping of the gradient list the optimizer is about to see (fp64, in place).
// norm = sqrt(sum over all tensors and elements of g^2); scale = max_norm / (norm + 1e-6),
// applied only when it is below 1.  Returns the scale that was applied (1 if none).
double gac_oracle_clip(int32_t n_tensors, double* const* g, const int64_t* numel,
                       double max_norm, double* norm_out) {
  double sq = 0.0;
  for (int32_t j = 0; j < n_tensors; ++j)
    for (int64_t i = 0; i < numel[j]; ++i) sq += g[j][i] * g[j][i];
  const double norm = std::sqrt(sq);
  if (norm_out != nullptr) *norm_out = norm;
  double scale = max_norm / (norm + 1e-6);
  if (!(scale < 1.0)) return 1.0;
  for (int32_t j = 0; j < n_tensors; ++j)
    for (int64_t i = 0; i < numel[j]; ++i) g[j][i] *= scale;
  return scale;
}

// Table 3 statistics of a run's cosines c_1 .. c_n: over the updates AFTER the first
// `burn_in` ones, the q-quantile of |c_t| (linear interpolation between order statistics
// at position (m-1) q, m = number of values), the maximum of |c_t| and the fraction with
// |c_t| <= c_low.  NaN entries (non-finite steps) are left out.  out = {quantile, max,
// fraction, m}; with m = 0 the first three are 0.
void gac_oracle_alignment_stats(const double* c, int64_t n, int64_t burn_in, double c_low,
                                double q, double out[4]) {
  std::vector<double> a;
  for (int64_t t = burn_in; t < n; ++t)
    if (!std::isnan(c[t])) a.push_back(std::fabs(c[t]));
  out[0] = out[1] = out[2] = 0.0;
  out[3] = static_cast<double>(a.size());
  if (a.empty()) return;
  std::sort(a.begin(), a.end());
  const double pos = (static_cast<double>(a.size()) - 1.0) * q;
  const size_t lo = static_cast<size_t>(std::floor(pos));
  const size_t hi = std::min(lo + 1, a.size() - 1);
  out[0] = a[lo] + (a[hi] - a[lo]) * (pos - static_cast<double>(lo));
  out[1] = a.back();
  int64_t inside = 0;
  for (double x : a) inside += (x <= c_low) ? 1 : 0;
  out[2] = static_cast<double>(inside) / static_cast<double>(a.size());
}

// Regime counts of a run's cosines c_1 .. c_n under a threshold pair: the rule of
// Section 4.2 (safe if |c| <= c_low, violation if |c| >= c_high, projection between) applied
// to every c_t after the first `burn_in` updates; NaN entries (non-finite steps) are left
// out.  counts = {safe, projected, skipped}.  Table 4 varies the pair around (0.05, 0.3).
void gac_oracle_regime_counts(const double* c, int64_t n, int64_t burn_in, double c_low,
                              double c_high, int64_t counts[3]) {
  counts[0] = counts[1] = counts[2] = 0;
  for (int64_t step = burn_in + 1; step <= n; ++step) {  // c[step - 1] is the cosine of update `step`
    const double mag = std::fabs(c[step - 1]);
    if (std::isnan(mag)) continue;
    int regime = ORACLE_PROJECT;
    if (mag <= c_low) regime = ORACLE_SAFE;
    else if (mag >= c_high) regime = ORACLE_SKIP;
    counts[regime] += 1;
  }
}

}  // extern "C"
