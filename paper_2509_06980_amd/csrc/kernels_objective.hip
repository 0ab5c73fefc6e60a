// Token-level masked GRPO objective, forward value (the loss the loss mask of Section 2.3.2 feeds;
// group sampling as in the multi-turn interaction example of Section 2.3).  The definition is the
// published GRPO one: group-normalised reward as the advantage of every sampled token of a
// trajectory, clipped importance ratio, and the non-negative KL estimator exp(d) - d - 1 with
// d = log pi_ref - log pi_new.  All sums are float64 and taken in a fixed order (no atomics).
#include "kernels.h"

namespace {

// One thread per trajectory: advantage within its group of G consecutive rewards, and its three
// accumulators (sum of terms, sum of KL estimates, number of tokens) cleared.
__global__ void grpo_advantage_kernel(const float* __restrict__ rewards, int n, int G, double eps_std,
                                      int ddof, double* __restrict__ adv, double* __restrict__ acc) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int g0 = i / G * G;
  double mean = 0.0;
  for (int j = 0; j < G; j++) mean += (double)rewards[g0 + j];
  mean /= (double)G;
  double var = 0.0;
  for (int j = 0; j < G; j++) {
    double d = (double)rewards[g0 + j] - mean;
    var += d * d;
  }
  double sd = sqrt(var / (double)(G - ddof));
  adv[i] = ((double)rewards[i] - mean) / (sd + eps_std);
  acc[3 * i] = 0.0;
  acc[3 * i + 1] = 0.0;
  acc[3 * i + 2] = 0.0;
}

// Sum of three per-thread values over a workgroup of 256, same order every time.
__device__ inline void block_sum3(double& a, double& b, double& c, double (*sh)[256]) {
  int t = threadIdx.x;
  sh[0][t] = a; sh[1][t] = b; sh[2][t] = c;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (t < w) {
      sh[0][t] += sh[0][t + w];
      sh[1][t] += sh[1][t + w];
      sh[2][t] += sh[2][t + w];
    }
    __syncthreads();
  }
  a = sh[0][0]; b = sh[1][0]; c = sh[2][0];
}

// One workgroup per segment (trajectory index, first row, end row) of the rows of this block of
// the pass: adds the segment's terms to the trajectory's accumulators.  A trajectory has at most
// one segment per launch and launches are stream-ordered, so the plain read-modify-write is safe.
__global__ __launch_bounds__(256) void grpo_terms_kernel(
    const float* __restrict__ lp, const float* __restrict__ old_lp, const float* __restrict__ ref_lp,
    const int32_t* __restrict__ use, const int32_t* __restrict__ segs, const double* __restrict__ adv,
    double clip_eps, double beta, double* __restrict__ acc) {
  __shared__ double sh[3][256];
  const int ti = segs[3 * blockIdx.x], k0 = segs[3 * blockIdx.x + 1], k1 = segs[3 * blockIdx.x + 2];
  const double A = adv[ti], lo = 1.0 - clip_eps, hi = 1.0 + clip_eps;
  double s = 0.0, skl = 0.0, cnt = 0.0;
  for (int k = k0 + threadIdx.x; k < k1; k += 256) {
    if (!use[k]) continue;
    double x = (double)lp[k];
    double rho = exp(x - (double)old_lp[k]);
    double cl = fmin(fmax(rho, lo), hi);
    double t = fmin(rho * A, cl * A);
    if (ref_lp) {
      double d = (double)ref_lp[k] - x;
      double k3 = exp(d) - d - 1.0;
      t -= beta * k3;
      skl += k3;
    }
    s += t;
    cnt += 1.0;
  }
  block_sum3(s, skl, cnt, sh);
  if (threadIdx.x == 0) {
    acc[3 * ti] += s;
    acc[3 * ti + 1] += skl;
    acc[3 * ti + 2] += cnt;
  }
}

// out[0] = mean over trajectories of (their mean term), out[1] = same for the KL estimate,
// out[2] = number of tokens that took part.
__global__ __launch_bounds__(256) void grpo_finish_kernel(const double* __restrict__ acc, int n,
                                                          double* __restrict__ out) {
  __shared__ double sh[3][256];
  double j = 0.0, kl = 0.0, cnt = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) {
    double c = acc[3 * i + 2];
    if (c > 0.0) {
      j += acc[3 * i] / c;
      kl += acc[3 * i + 1] / c;
      cnt += c;
    }
  }
  block_sum3(j, kl, cnt, sh);
  if (threadIdx.x == 0) {
    out[0] = n > 0 ? j / (double)n : 0.0;
    out[1] = n > 0 ? kl / (double)n : 0.0;
    out[2] = cnt;
  }
}

}  // namespace

void launch_grpo_advantages(hipStream_t s, const float* rewards, int n, int G, double eps_std, int ddof,
                            double* adv, double* acc) {
  if (n <= 0) return;
  grpo_advantage_kernel<<<(n + 63) / 64, 64, 0, s>>>(rewards, n, G, eps_std, ddof, adv, acc);
}

void launch_grpo_terms(hipStream_t s, const float* lp, const float* old_lp, const float* ref_lp,
                       const int32_t* use, const int32_t* segs, int nseg, const double* adv,
                       double clip_eps, double beta, double* acc) {
  if (nseg <= 0) return;
  grpo_terms_kernel<<<nseg, 256, 0, s>>>(lp, old_lp, ref_lp, use, segs, adv, clip_eps, beta, acc);
}

void launch_grpo_finish(hipStream_t s, const double* acc, int n, double* out) {
  grpo_finish_kernel<<<1, 256, 0, s>>>(acc, n, out);
}
