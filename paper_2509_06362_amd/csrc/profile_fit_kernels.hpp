// Profiler: least-squares fit of the throughput-decay function (Sec. IV-B, Eq. 1)
//   F(w) = T0 * (1 - delta * log(eps + w)),   w = min(B, W),
// to measured (w, throughput) samples of one parallelism strategy, and the per-token latency table
// 1 / F(b), b = 1 .. b_cap, that the scoring kernels read.
//
// For a fixed eps the model is linear in (T0, T0 * delta): with x = log(eps + w) it is the straight line
// y = alpha - beta * x, whose least-squares fit has the closed form below; what remains is a
// one-dimensional minimisation of the residual over eps.  That is done by nested grid search on
// log(eps): kFitGrid points between the bounds, keep the best (lowest index on ties), shrink the
// bounds to its two neighbours, kFitLevels times.  All arithmetic is binary64.  One block per
// strategy, one thread per grid point; samples are read from global memory (they are few).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace maaso {

constexpr int kFitGrid = 256;
constexpr int kFitLevels = 10;

struct FitArgs {
  const uint32_t* offsets;  // [n_tp + 1] samples of strategy t are [offsets[t], offsets[t+1])
  const float* level;       // [N] w = min(B, W) of the sample, >= 1
  const float* thr;         // [N] measured throughput, tokens/s
  uint32_t b_cap;
  double log_eps_lo, log_eps_hi;
  double* params;           // [n_tp][4] T0, delta, eps, residual sum of squares
  float* tbt;               // [n_tp][b_cap + 1]; column 0 is NaN
  uint32_t* bad;            // [1] set to 1 when a strategy cannot be fitted or F(b) <= 0 for some b
};

// Residual sum of squares of the best straight line through (log(eps + w_i), y_i), and the line.
struct LineFit {
  double alpha, beta, sse;
  bool ok;
};

__device__ inline LineFit fit_line(const float* __restrict__ w, const float* __restrict__ y, uint32_t n,
                                   double eps) {
  double sx = 0.0, sy = 0.0;
  for (uint32_t i = 0; i < n; ++i) {
    sx += log(eps + (double)w[i]);
    sy += (double)y[i];
  }
  const double mx = sx / (double)n, my = sy / (double)n;
  double sxx = 0.0, sxy = 0.0, syy = 0.0;
  for (uint32_t i = 0; i < n; ++i) {
    const double dx = log(eps + (double)w[i]) - mx, dy = (double)y[i] - my;
    sxx += dx * dx;
    sxy += dx * dy;
    syy += dy * dy;
  }
  LineFit f;
  f.ok = sxx > 0.0;
  const double slope = f.ok ? sxy / sxx : 0.0;
  f.beta = -slope;
  f.alpha = my - slope * mx;
  f.sse = syy - slope * sxy;
  return f;
}

__global__ __launch_bounds__(kFitGrid) void profile_fit_kernel(const FitArgs a) {
  __shared__ double s_sse[kFitGrid];
  __shared__ double s_lo, s_hi;
  const uint32_t t = blockIdx.x, tid = threadIdx.x;
  const uint32_t o0 = a.offsets[t], o1 = a.offsets[t + 1];
  const uint32_t n = o1 > o0 ? o1 - o0 : 0u;
  const float* w = a.level + o0;
  const float* y = a.thr + o0;
  float* row = a.tbt + (size_t)t * (a.b_cap + 1u);
  double* out = a.params + (size_t)t * 4u;
  if (n < 3u) {  // three parameters need three samples
    if (tid == 0) { *a.bad = 1u; out[0] = out[1] = out[2] = out[3] = __builtin_nan(""); }
    for (uint32_t b = tid; b <= a.b_cap; b += kFitGrid) row[b] = __builtin_nanf("");
    return;
  }
  if (tid == 0) { s_lo = a.log_eps_lo; s_hi = a.log_eps_hi; }
  __syncthreads();
  for (int level = 0; level < kFitLevels; ++level) {
    const double lo = s_lo, hi = s_hi;
    const double le = lo + (hi - lo) * ((double)tid / (double)(kFitGrid - 1));
    const LineFit f = fit_line(w, y, n, exp(le));
    s_sse[tid] = f.ok ? f.sse : __builtin_inf();
    __syncthreads();
    if (tid == 0) {
      int best = 0;
      for (int i = 1; i < kFitGrid; ++i)
        if (s_sse[i] < s_sse[best]) best = i;
      const int bl = best > 0 ? best - 1 : 0, bh = best < kFitGrid - 1 ? best + 1 : kFitGrid - 1;
      s_lo = lo + (hi - lo) * ((double)bl / (double)(kFitGrid - 1));
      s_hi = lo + (hi - lo) * ((double)bh / (double)(kFitGrid - 1));
    }
    __syncthreads();
  }
  // the centre of the last bracket is the answer
  const double eps = exp(0.5 * (s_lo + s_hi));
  const LineFit f = fit_line(w, y, n, eps);
  const double t0 = f.alpha, delta = f.beta / f.alpha;
  if (tid == 0) { out[0] = t0; out[1] = delta; out[2] = eps; out[3] = f.sse; }
  bool bad = !f.ok || !(t0 > 0.0);
  for (uint32_t b = tid; b <= a.b_cap; b += kFitGrid) {
    if (b == 0u) { row[0] = __builtin_nanf(""); continue; }
    const double fb = t0 * (1.0 - delta * log(eps + (double)b));
    if (!(fb > 0.0)) bad = true;
    row[b] = (float)(1.0 / fb);
  }
  if (bad) *a.bad = 1u;
}

}  // namespace maaso
