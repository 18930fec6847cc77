// Error-guided Budgeted Calibration (Sec. 4.3): the two computations that turn measured
// velocities into per-head thresholds.
//
//  heart_ebc_band_error   the frequency-weighted velocity error of Eq. 6 on the GPU.
//    The four bands of the appendix (after fftshift a frequency is low along an axis of
//    length n when it lies within floor(n/4) of the centre) are products of per-axis
//    low / high sets, and the low set {-r..r} is symmetric, so its indicator in the
//    frequency domain is a real orthogonal projection P in the signal domain: a circular
//    convolution with the Dirichlet kernel p[d] = (1/n)(1 + 2 sum_{f=1..r} cos(2 pi f d / n)).
//    By Parseval, with n_tot = T*Y*X and the unnormalised transform of the definition,
//        E_LL = n_tot |Pt Py Px e|^2            E_LH = n_tot (|Pt e|^2 - |Pt Py Px e|^2)
//        E_HL = n_tot (|Py Px e|^2 - |Pt Py Px e|^2)
//        E_HH = n_tot (|e|^2 - |Pt e|^2 - |Py Px e|^2 + |Pt Py Px e|^2)
//    and the denominator is n_tot |dense|^2 + epsilon.  No transform is computed: three
//    circular convolutions (n^2 work per line, n <= a few hundred) in fp64 and four
//    deterministic reductions.  A calibration run evaluates this once per (head,
//    candidate, prompt-step), off the serving path.
//
//  heart_ebc_select       the one-candidate-per-head selection of Eq. 5 (minimum summed
//    error under a mean-sparsity budget), solved exactly on the host: linear relaxation of
//    the multiple-choice knapsack (per-head lower convex hulls, increments in order of
//    error per unit of sparsity) as the bound of a depth-first branch and bound on the one
//    head the relaxation leaves fractional.  Replaces the generic integer-program solver
//    the paper uses.
#include <algorithm>
#include <cmath>
#include <vector>

#include "heart_internal.h"

namespace heart {

constexpr int kEbcThreads = 256;
constexpr int kEbcMaxAxis = 1024;   // longest axis the convolution kernel stages in LDS
constexpr int kEbcPartials = 1024;  // partial sums per reduction

// p[d], d = 0..n-1, of the low-pass projection along an axis of length n
__global__ void ebc_dirichlet_kernel(int n, double *__restrict__ p) {
  const int r = n / 4;
  for (int d = blockIdx.x * blockDim.x + threadIdx.x; d < n; d += gridDim.x * blockDim.x) {
    double s = 1.0;
    for (int f = 1; f <= r; ++f) {
      // reduce f*d modulo n in integers so that the argument of cospi stays in [0, 2)
      const long long m = ((long long)f * d) % n;
      s += 2.0 * cospi(2.0 * (double)m / (double)n);
    }
    p[d] = s / (double)n;
  }
}

// out[o, i, s] = sum_j p[(i - j) mod n] * in[o, j, s]   for a tensor viewed as [outer][n][inner]
template <typename TIn>
__global__ __launch_bounds__(kEbcThreads) void ebc_project_kernel(
    const TIn *__restrict__ in, double *__restrict__ out, const double *__restrict__ p, int n,
    long long inner, long long total) {
  __shared__ double sp[kEbcMaxAxis];
  for (int d = threadIdx.x; d < n; d += kEbcThreads) sp[d] = p[d];
  __syncthreads();
  for (long long e = (long long)blockIdx.x * kEbcThreads + threadIdx.x; e < total;
       e += (long long)gridDim.x * kEbcThreads) {
    const long long s = e % inner;
    const long long oi = e / inner;
    const int i = (int)(oi % n);
    const long long o = oi / n;
    const TIn *line = in + o * n * inner + s;
    double acc = 0.0;
    int d = i;  // (i - j) mod n for j = 0
    for (int j = 0; j < n; ++j) {
      acc = fma(sp[d], (double)line[(long long)j * inner], acc);
      d = d == 0 ? n - 1 : d - 1;
    }
    out[e] = acc;
  }
}

// partial[b] = sum of squares of the elements block b owns (fixed assignment and order)
template <typename TIn>
__global__ __launch_bounds__(kEbcThreads) void ebc_sumsq_kernel(const TIn *__restrict__ x,
                                                                long long total,
                                                                double *__restrict__ partial) {
  __shared__ double red[kEbcThreads];
  double acc = 0.0;
  for (long long e = (long long)blockIdx.x * kEbcThreads + threadIdx.x; e < total;
       e += (long long)gridDim.x * kEbcThreads) {
    const double v = (double)x[e];
    acc = fma(v, v, acc);
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kEbcThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// sums[k] = sum of the kEbcPartials partials of reduction k (k = 0..4: |e|^2, |Pt e|^2,
// |Py Px e|^2, |Pt Py Px e|^2, |dense|^2), then the band energies and the weighted error
__global__ __launch_bounds__(kEbcThreads) void ebc_finish_kernel(const double *__restrict__ partials,
                                                                 double n_tot, double w0, double w1,
                                                                 double w2, double w3, double epsilon,
                                                                 double *__restrict__ out) {
  __shared__ double red[kEbcThreads];
  __shared__ double sums[5];
  for (int k = 0; k < 5; ++k) {
    double acc = 0.0;
    for (int i = threadIdx.x; i < kEbcPartials; i += kEbcThreads) acc += partials[k * kEbcPartials + i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = kEbcThreads / 2; s > 0; s >>= 1) {
      if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
      __syncthreads();
    }
    if (threadIdx.x == 0) sums[k] = red[0];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double tot = sums[0], a = sums[1], b = sums[2], c = sums[3];
    const double ll = n_tot * c, lh = n_tot * (a - c), hl = n_tot * (b - c),
                 hh = n_tot * (tot - a - b + c);
    const double den = n_tot * sums[4] + epsilon;
    out[0] = (w0 * ll + w1 * lh + w2 * hl + w3 * hh) / den;
    out[1] = ll;
    out[2] = lh;
    out[3] = hl;
    out[4] = hh;
    out[5] = n_tot * sums[4];
  }
}

static size_t ebc_workspace_doubles(long long total, int T, int Y, int X) {
  return 2 * (size_t)total + (size_t)(T + Y + X) + 5 * (size_t)kEbcPartials;
}

int launch_ebc_band_error(long long C, int T, int Y, int X, const float *err, const float *dense,
                          const double *w, double epsilon, double *ws, double *out,
                          hipStream_t st) {
  const long long total = C * T * Y * X;
  double *bufa = ws, *bufb = ws + total;
  double *pt = bufb + total, *py = pt + T, *px = py + Y;
  double *partials = px + X;
  const int grid = (int)std::min<long long>((total + kEbcThreads - 1) / kEbcThreads, 4096);
  hipLaunchKernelGGL(ebc_dirichlet_kernel, dim3(1), dim3(256), 0, st, T, pt);
  hipLaunchKernelGGL(ebc_dirichlet_kernel, dim3(1), dim3(256), 0, st, Y, py);
  hipLaunchKernelGGL(ebc_dirichlet_kernel, dim3(1), dim3(256), 0, st, X, px);
  // |e|^2 and |dense|^2
  hipLaunchKernelGGL(ebc_sumsq_kernel<float>, dim3(kEbcPartials), dim3(kEbcThreads), 0, st, err,
                     total, partials + 0 * kEbcPartials);
  hipLaunchKernelGGL(ebc_sumsq_kernel<float>, dim3(kEbcPartials), dim3(kEbcThreads), 0, st, dense,
                     total, partials + 4 * kEbcPartials);
  // Pt e -> bufa
  hipLaunchKernelGGL(ebc_project_kernel<float>, dim3(grid), dim3(kEbcThreads), 0, st, err, bufa, pt,
                     T, (long long)Y * X, total);
  hipLaunchKernelGGL(ebc_sumsq_kernel<double>, dim3(kEbcPartials), dim3(kEbcThreads), 0, st, bufa,
                     total, partials + 1 * kEbcPartials);
  // Px e -> bufa, Py Px e -> bufb
  hipLaunchKernelGGL(ebc_project_kernel<float>, dim3(grid), dim3(kEbcThreads), 0, st, err, bufa, px,
                     X, 1LL, total);
  hipLaunchKernelGGL(ebc_project_kernel<double>, dim3(grid), dim3(kEbcThreads), 0, st, bufa, bufb,
                     py, Y, (long long)X, total);
  hipLaunchKernelGGL(ebc_sumsq_kernel<double>, dim3(kEbcPartials), dim3(kEbcThreads), 0, st, bufb,
                     total, partials + 2 * kEbcPartials);
  // Pt Py Px e -> bufa
  hipLaunchKernelGGL(ebc_project_kernel<double>, dim3(grid), dim3(kEbcThreads), 0, st, bufb, bufa,
                     pt, T, (long long)Y * X, total);
  hipLaunchKernelGGL(ebc_sumsq_kernel<double>, dim3(kEbcPartials), dim3(kEbcThreads), 0, st, bufa,
                     total, partials + 3 * kEbcPartials);
  hipLaunchKernelGGL(ebc_finish_kernel, dim3(1), dim3(kEbcThreads), 0, st, partials,
                     (double)T * Y * X, w[0], w[1], w[2], w[3], epsilon, out);
  return check_launch("ebc kernels");
}

// ---------------------------------------------------------------------------------------
// Selection (host).  Heads i = 0..n-1, candidates c = 0..k-1 with error E[i*k+c] and
// sparsity S[i*k+c]; minimise sum E subject to sum S >= need.
namespace {

struct Inc {       // one step along a head's lower convex hull
  int head, to;    // candidate reached by taking this step (and all earlier ones of the head)
  double ds, de;   // gain in sparsity (> 0) and cost in error (>= 0 after dominance pruning)
};

struct Solver {
  int n, k;
  const double *E, *S;
  double need;
  std::vector<int> base;               // per head: candidate of least error (ties: most sparse)
  std::vector<std::vector<int>> hull;  // per head: hull candidates after base, sparsity ascending
  std::vector<Inc> incs;               // all hull steps, cheapest error per sparsity first
  std::vector<int> fixed, best;
  std::vector<char> removed;           // [n*k] candidates proved useless by their reduced cost
  double best_e;
  long long nodes;

  double e(int i, int c) const { return E[(size_t)i * k + c]; }
  double s(int i, int c) const { return S[(size_t)i * k + c]; }

  bool ok(int i, int c) const { return !removed[(size_t)i * k + c]; }

  void build() {
    base.assign(n, 0);
    hull.assign(n, {});
    incs.clear();
    for (int i = 0; i < n; ++i) {
      int b = -1;
      for (int c = 0; c < k; ++c)
        if (ok(i, c) && (b < 0 || e(i, c) < e(i, b) || (e(i, c) == e(i, b) && s(i, c) > s(i, b)))) b = c;
      base[i] = b;  // (at least one candidate of every head survives the reduction)
      // candidates that add sparsity over the base, by sparsity; keep the lower convex hull
      std::vector<int> cand;
      for (int c = 0; c < k; ++c)
        if (ok(i, c) && s(i, c) > s(i, b)) cand.push_back(c);
      std::sort(cand.begin(), cand.end(), [&](int a, int c2) {
        return s(i, a) < s(i, c2) || (s(i, a) == s(i, c2) && e(i, a) < e(i, c2));
      });
      std::vector<int> h = {b};
      for (int c : cand) {
        if (s(i, c) == s(i, h.back())) continue;  // same sparsity, more error
        while (h.size() >= 2) {
          const int p1 = h[h.size() - 2], p2 = h.back();
          // drop p2 if it lies on or above the segment p1 -> c
          const double cross = (s(i, p2) - s(i, p1)) * (e(i, c) - e(i, p1)) -
                               (e(i, p2) - e(i, p1)) * (s(i, c) - s(i, p1));
          if (cross <= 0.0) h.pop_back(); else break;
        }
        h.push_back(c);
      }
      for (size_t j = 1; j < h.size(); ++j) {
        hull[i].push_back(h[j]);
        incs.push_back({i, h[j], s(i, h[j]) - s(i, h[j - 1]), e(i, h[j]) - e(i, h[j - 1])});
      }
    }
    std::stable_sort(incs.begin(), incs.end(),
                     [](const Inc &a, const Inc &b) { return a.de * b.ds < b.de * a.ds; });
  }

  // Relaxation with some heads fixed.  Returns the bound; `frac_head` is the head whose step
  // was taken partially (-1 if the relaxed solution is integral), `sol` the integral part.
  bool relax(double &bound, int &frac_head, std::vector<int> &sol, double &sol_e, double &sol_s,
             double *lambda = nullptr) {
    double se = 0.0, ss = 0.0;
    sol.assign(n, 0);
    for (int i = 0; i < n; ++i) {
      sol[i] = fixed[i] >= 0 ? fixed[i] : base[i];
      se += e(i, sol[i]);
      ss += s(i, sol[i]);
    }
    frac_head = -1;
    if (lambda) *lambda = 0.0;
    if (ss >= need) { bound = se; sol_e = se; sol_s = ss; return true; }
    for (const Inc &in : incs) {
      if (fixed[in.head] >= 0) continue;
      if (ss + in.ds >= need) {
        // this step reaches the budget: fractional unless it lands exactly on it
        const double f = (need - ss) / in.ds;
        bound = se + f * in.de;
        frac_head = in.head;
        if (lambda) *lambda = in.de / in.ds;
        // integral completion: take the whole step (feasible)
        sol[in.head] = in.to;
        sol_e = se + in.de;
        sol_s = ss + in.ds;
        return true;
      }
      sol[in.head] = in.to;
      se += in.de;
      ss += in.ds;
    }
    return false;  // budget out of reach
  }

  // Single-head moves that lower the error and keep the budget, best first, until none is left.
  void improve(std::vector<int> &sol, double &sol_e, double &sol_s) const {
    for (;;) {
      int bi = -1, bc = -1;
      double gain = 0.0;
      for (int i = 0; i < n; ++i) {
        if (fixed[i] >= 0) continue;
        const double e0 = e(i, sol[i]), s0 = s(i, sol[i]);
        for (int c = 0; c < k; ++c) {
          if (!ok(i, c)) continue;
          const double de = e0 - e(i, c);
          if (de > gain && sol_s - s0 + s(i, c) >= need) gain = de, bi = i, bc = c;
        }
      }
      if (bi < 0) return;
      sol_e -= gain;
      sol_s += s(bi, bc) - s(bi, sol[bi]);
      sol[bi] = bc;
    }
  }

  static constexpr long long kNodeLimit = 2000000;
  void search() {
    if (++nodes > kNodeLimit) return;
    double bound, se, ss;
    int fh;
    std::vector<int> sol;
    if (!relax(bound, fh, sol, se, ss)) return;
    if (bound >= best_e) return;
    if (se < best_e + (best_e - bound)) improve(sol, se, ss);  // worth polishing
    if (se < best_e) { best_e = se; best = sol; }  // the integral completion is feasible
    if (fh < 0 || bound >= best_e) return;          // relaxed solution was integral
    // branch on the fractional head: each of its candidates in turn, most promising first
    std::vector<int> order(k);
    for (int c = 0; c < k; ++c) order[c] = c;
    std::sort(order.begin(), order.end(), [&](int a, int b) { return e(fh, a) < e(fh, b); });
    for (int c : order) {
      if (!ok(fh, c)) continue;
      fixed[fh] = c;
      search();
    }
    fixed[fh] = -1;
  }
};

}  // namespace

int ebc_select_host(int n, int k, const double *E, const double *S, double s_min, int *choice,
                    double *total_error, long long *nodes) {
  Solver sv;
  sv.n = n; sv.k = k; sv.E = E; sv.S = S;
  sv.need = s_min * (double)n - 1e-12 * (double)n;
  sv.removed.assign((size_t)n * k, 0);
  sv.build();
  sv.fixed.assign(n, -1);
  sv.best_e = INFINITY;
  sv.nodes = 0;
  {
    // Root: relaxation, incumbent, and reduced-cost fixing.  With the multiplier lambda of
    // the relaxation, any selection that uses candidate (i, c) costs at least
    //   bound + (E_ic - lambda S_ic) - min_c' (E_ic' - lambda S_ic'),
    // so candidates for which that is not below the incumbent can be discarded.  The gap of
    // this problem is at most one hull step, so almost every head is left with one candidate.
    double bound, se, ss, lambda;
    int fh;
    std::vector<int> sol;
    if (sv.relax(bound, fh, sol, se, ss, &lambda)) {
      sv.improve(sol, se, ss);
      sv.best_e = se;
      sv.best = sol;
      if (fh >= 0) {
        const double gap = se - bound;
        for (int i = 0; i < n; ++i) {
          double lo = INFINITY;
          for (int c = 0; c < k; ++c) lo = std::min(lo, sv.e(i, c) - lambda * sv.s(i, c));
          for (int c = 0; c < k; ++c)
            if (sv.e(i, c) - lambda * sv.s(i, c) - lo >= gap + 1e-15 * std::fabs(se) && c != sol[i])
              sv.removed[(size_t)i * k + c] = 1;
        }
        sv.build();
        sv.search();
      }
    }
  }
  if (nodes) *nodes = sv.nodes;
  if (sv.best.empty()) return 1;  // infeasible
  if (sv.nodes > Solver::kNodeLimit) return 2;  // optimality not proved within the node limit
  for (int i = 0; i < n; ++i) choice[i] = sv.best[i];
  double tot = 0.0;
  for (int i = 0; i < n; ++i) tot += sv.e(i, sv.best[i]);
  *total_error = tot;
  return 0;
}

size_t ebc_workspace_bytes(long long C, int T, int Y, int X) {
  return ebc_workspace_doubles(C * T * Y * X, T, Y, X) * sizeof(double);
}

}  // namespace heart
