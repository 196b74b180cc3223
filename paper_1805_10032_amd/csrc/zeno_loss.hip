// Loss head and score combine of the Stochastic Descendant Score (Definition 2).
//
// The layer kernels deliver, for the output layer, the pre-activations at x (Z0)
// and, per candidate, their change dZ_i caused by moving to x - gamma u_i.
// Per sample k this file forms f(x - gamma u_i; z_k) - f(x; z_k) in fp64
// directly from (Z0, dZ_i), then
//     score_i = -(1/n_r) sum_k diff_ik - rho ||u_i||^2 .
#include "zeno_internal.h"

namespace zeno {

namespace {

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ inline double wave_max(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, 64));
  return v;
}

// One wave per (sample, candidate).  Softmax cross-entropy:
//   diff = logsumexp(z0 + dz) - logsumexp(z0) - dz[label]
// squared loss (output width 1):
//   diff = 1/2 (z0 + dz - y)^2 - 1/2 (z0 - y)^2 = dz ((z0 - y) + dz/2).
// A NaN anywhere in dz reaches the sum of exponentials and makes diff NaN.
__global__ __launch_bounds__(64) void loss_diff_kernel(const float* __restrict__ Z0, const float* __restrict__ dZ,
                                                       const int32_t* __restrict__ labels,
                                                       const float* __restrict__ targets, int loss, int n_r_total,
                                                       int chunk_begin, int chunk_rows, int C,
                                                       double* __restrict__ sample_diff) {
  const int kk = blockIdx.x, i = blockIdx.y, lane = threadIdx.x;
  const float* z0 = Z0 + (long long)kk * C;
  const float* dz = dZ + ((long long)i * chunk_rows + kk) * C;
  double diff;
  if (loss == ZENO_LOSS_SQUARED) {
    const double z = (double)z0[0], t = (double)dz[0], y = (double)targets[chunk_begin + kk];
    diff = t * ((z - y) + 0.5 * t);
  } else {
    double m0 = -__builtin_inf(), m1 = -__builtin_inf();
    for (int c = lane; c < C; c += 64) {
      const double a = (double)z0[c], b = a + (double)dz[c];
      m0 = fmax(m0, a);
      m1 = fmax(m1, b);
    }
    m0 = wave_max(m0);
    m1 = wave_max(m1);
    double s0 = 0.0, s1 = 0.0;
    for (int c = lane; c < C; c += 64) {
      const double a = (double)z0[c], b = a + (double)dz[c];
      s0 += exp(a - m0);
      s1 += exp(b - m1);
    }
    s0 = wave_sum(s0);
    s1 = wave_sum(s1);
    // a label outside [0, C) has no logit: the sample's loss difference becomes NaN (and with it
    // every score) instead of reading past the row
    const int y = labels[chunk_begin + kk];
    const double dzy = (y >= 0 && y < C) ? (double)dz[y] : __builtin_nan("");
    diff = ((m1 + log(s1)) - (m0 + log(s0))) - dzy;
  }
  if (lane == 0) sample_diff[(long long)i * n_r_total + chunk_begin + kk] = diff;
}

// One wave per candidate: mean over the n_r samples, sum of the partial squared
// norms, and the three-term combine, all in fp64, rounded once to fp32.
// A candidate's partial norms lie P_stride apart, of which the first P are in use.
__global__ __launch_bounds__(64) void score_combine_kernel(const double* __restrict__ sample_diff,
                                                           const double* __restrict__ norm_partials, int P_stride, int P,
                                                           int n_r_total, float rho, float* __restrict__ scores) {
  const int i = blockIdx.x, lane = threadIdx.x;
  double sd = 0.0, sn = 0.0;
  for (int k = lane; k < n_r_total; k += 64) sd += sample_diff[(long long)i * n_r_total + k];
  for (int p = lane; p < P; p += 64) sn += norm_partials[(long long)i * P_stride + p];
  sd = wave_sum(sd);
  sn = wave_sum(sn);
  if (lane == 0) scores[i] = (float)(-(sd / (double)n_r_total) - (double)rho * sn);
}

}  // namespace

hipError_t launch_loss(const float* Z0, const float* dZ, const int32_t* labels, const float* targets, int loss,
                       int m, int n_r_total, int chunk_begin, int chunk_rows, int C, double* sample_diff,
                       hipStream_t stream) {
  hipLaunchKernelGGL(loss_diff_kernel, dim3(chunk_rows, m), dim3(64), 0, stream, Z0, dZ, labels, targets, loss,
                     n_r_total, chunk_begin, chunk_rows, C, sample_diff);
  return hipGetLastError();
}

hipError_t launch_score_combine_strided(const double* sample_diff, const double* norm_partials, int P_stride, int P,
                                        int m, int n_r_total, float rho, float* scores, hipStream_t stream) {
  hipLaunchKernelGGL(score_combine_kernel, dim3(m), dim3(64), 0, stream, sample_diff, norm_partials, P_stride, P,
                     n_r_total, rho, scores);
  return hipGetLastError();
}

hipError_t launch_score_combine(const double* sample_diff, const double* norm_partials, int P, int m,
                                int n_r_total, float rho, float* scores, hipStream_t stream) {
  return launch_score_combine_strided(sample_diff, norm_partials, P, P, m, n_r_total, rho, scores, stream);
}

}  // namespace zeno
