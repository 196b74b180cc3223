// Marginal median (Definition 4): for every coordinate j the one-dimensional
// median of the m values G[0][j] .. G[m-1][j].  Each lane owns one column,
// keeps its m values in registers as order-preserving integer keys, and sorts
// them with a fully unrolled bitonic network of compile-time width P >= m.
#include <limits.h>

#include "zeno_internal.h"

namespace zeno {

namespace {

constexpr int kThreads = 256;

// Monotone map float -> int32: integer order equals the total order
// -inf < ... < -0 < +0 < ... < +inf < NaN (every NaN becomes the top key).
__device__ inline int float_key(float f) {
  int k = __float_as_int(f);
  k ^= (k >> 31) & 0x7fffffff;
  return (f != f) ? INT_MAX : k;
}
__device__ inline float key_float(int k) {
  return __int_as_float(k ^ ((k >> 31) & 0x7fffffff));
}

template <int P>
__global__ __launch_bounds__(kThreads) void median_kernel(const float* __restrict__ G, int m, long long d,
                                                          float* __restrict__ out) {
  const long long stride = (long long)gridDim.x * kThreads;
  const int lo = (m - 1) / 2, hi = m / 2;
  for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < d; j += stride) {
    int v[P];
#pragma unroll
    for (int i = 0; i < P; ++i) v[i] = (i < m) ? float_key(G[(long long)i * d + j]) : INT_MAX;
#pragma unroll
    for (int k = 2; k <= P; k <<= 1) {
#pragma unroll
      for (int s = k >> 1; s > 0; s >>= 1) {
#pragma unroll
        for (int i = 0; i < P; ++i) {
          const int l = i ^ s;
          if (l > i) {
            const int a = v[i], c = v[l];
            const int mn = a < c ? a : c, mx = a < c ? c : a;
            const bool up = (i & k) == 0;
            v[i] = up ? mn : mx;
            v[l] = up ? mx : mn;
          }
        }
      }
    }
    int ka = 0, kb = 0;
#pragma unroll
    for (int i = 0; i < P; ++i) {
      ka = (i == lo) ? v[i] : ka;
      kb = (i == hi) ? v[i] : kb;
    }
    const float fa = key_float(ka), fb = key_float(kb);
    out[j] = (lo == hi) ? fa : (float)(0.5 * ((double)fa + (double)fb));
  }
}

template <int P>
hipError_t launch_p(const float* G, int m, long long d, float* out, hipStream_t stream) {
  long long want = (d + kThreads - 1) / kThreads;
  int grid = (int)(want < 1 ? 1 : (want > 256 * 32 ? 256 * 32 : want));
  hipLaunchKernelGGL(median_kernel<P>, dim3(grid), dim3(kThreads), 0, stream, G, m, d, out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_median(const float* G, int m, long long d, float* out, hipStream_t stream) {
  if (m <= 2) return launch_p<2>(G, m, d, out, stream);
  if (m <= 4) return launch_p<4>(G, m, d, out, stream);
  if (m <= 8) return launch_p<8>(G, m, d, out, stream);
  if (m <= 16) return launch_p<16>(G, m, d, out, stream);
  if (m <= 32) return launch_p<32>(G, m, d, out, stream);
  if (m <= 64) return launch_p<64>(G, m, d, out, stream);
  return launch_p<128>(G, m, d, out, stream);
}

}  // namespace zeno
