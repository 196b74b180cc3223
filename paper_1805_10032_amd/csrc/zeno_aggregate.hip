// Selection of the m-b highest scores and the average of the selected rows
// (Definition 3, Zeno_b), and the Mean baseline (Section 6.1.1) as the b = 0
// case without scores.  One streaming pass over the selected rows of G.
#include "zeno_internal.h"

namespace zeno {

namespace {

constexpr int kThreads = 256;
constexpr int kRowBatch = 8;  // rows whose loads are in flight together per thread

// Every workgroup redoes the selection from the m scores (m <= 1024, a few
// thousand compares) instead of waiting for a separate launch: rank_i = number
// of candidates that beat i under (score descending, index ascending), NaN
// scores ranking as -inf; i is chosen iff rank_i < m-b.  The list is built in
// ascending index order so that every workgroup sums rows in the same order.
__device__ void select_rows(const float* __restrict__ scores, int m, int n_sel, float* key, int* flag,
                            int* sel_list, int32_t* selected_out) {
  const int tid = threadIdx.x;
  for (int i = tid; i < m; i += kThreads) {
    float s = scores[i];
    key[i] = (s != s) ? -__builtin_inff() : s;
  }
  __syncthreads();
  for (int i = tid; i < m; i += kThreads) {
    const float si = key[i];
    int rank = 0;
    for (int j = 0; j < m; ++j) {
      const float sj = key[j];
      rank += (sj > si) || (sj == si && j < i);
    }
    flag[i] = rank < n_sel;
  }
  __syncthreads();
  for (int i = tid; i < m; i += kThreads) {
    if (flag[i]) {
      int pos = 0;
      for (int j = 0; j < i; ++j) pos += flag[j];
      sel_list[pos] = i;
      if (selected_out != nullptr) selected_out[pos] = i;
    }
  }
  __syncthreads();
}

template <bool ALL>
__global__ __launch_bounds__(kThreads) void masked_average_kernel(const float* __restrict__ G,
                                                                  const float* __restrict__ scores, int m,
                                                                  long long d, long long ldg, int b,
                                                                  float* __restrict__ out,
                                                                  int32_t* __restrict__ selected) {
  __shared__ float key[ZENO_MAX_CANDIDATES];
  __shared__ int flag[ZENO_MAX_CANDIDATES];
  __shared__ int sel_list[ZENO_MAX_CANDIDATES];
  const int n_sel = ALL ? m : m - b;
  if (!ALL) select_rows(scores, m, n_sel, key, flag, sel_list, blockIdx.x == 0 ? selected : nullptr);

  const double n = (double)n_sel;
  const long long n_vec = d / 4;
  const long long stride = (long long)gridDim.x * kThreads;
  for (long long c = (long long)blockIdx.x * kThreads + threadIdx.x; c < n_vec; c += stride) {
    const float* col = G + c * 4;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    int s = 0;
    for (; s + kRowBatch <= n_sel; s += kRowBatch) {
      f32x4 v[kRowBatch];
#pragma unroll
      for (int t = 0; t < kRowBatch; ++t) {
        const long long row = ALL ? (s + t) : sel_list[s + t];
        v[t] = load_stream4(col + row * ldg);
      }
#pragma unroll
      for (int t = 0; t < kRowBatch; ++t) {
        a0 += (double)v[t][0];
        a1 += (double)v[t][1];
        a2 += (double)v[t][2];
        a3 += (double)v[t][3];
      }
    }
    for (; s < n_sel; ++s) {
      const long long row = ALL ? s : sel_list[s];
      const f32x4 v = load_stream4(col + row * ldg);
      a0 += (double)v[0];
      a1 += (double)v[1];
      a2 += (double)v[2];
      a3 += (double)v[3];
    }
    f4u r;
    r.x = (float)(a0 / n);
    r.y = (float)(a1 / n);
    r.z = (float)(a2 / n);
    r.w = (float)(a3 / n);
    *reinterpret_cast<f4u*>(out + c * 4) = r;
  }
  // d mod 4 trailing columns
  if (blockIdx.x == 0) {
    for (long long j = n_vec * 4 + threadIdx.x; j < d; j += kThreads) {
      double a = 0.0;
      for (int s = 0; s < n_sel; ++s) {
        const long long row = ALL ? s : sel_list[s];
        a += (double)G[row * ldg + j];
      }
      out[j] = (float)(a / n);
    }
  }
}

}  // namespace

hipError_t launch_masked_average(const float* G, long long ldg, const float* scores, int m, long long d, int b,
                                 float* out, int32_t* selected, hipStream_t stream) {
  long long n_vec = d / 4;
  long long want = (n_vec + kThreads - 1) / kThreads;
  int grid = (int)(want < 1 ? 1 : (want > 256 * 16 ? 256 * 16 : want));
  if (scores == nullptr) {
    hipLaunchKernelGGL(masked_average_kernel<true>, dim3(grid), dim3(kThreads), 0, stream, G, scores, m, d, ldg,
                       0, out, selected);
  } else {
    hipLaunchKernelGGL(masked_average_kernel<false>, dim3(grid), dim3(kThreads), 0, stream, G, scores, m, d, ldg,
                       b, out, selected);
  }
  return hipGetLastError();
}

}  // namespace zeno
