// Marginal median (Definition 4): for every coordinate j the one-dimensional
// median of the m values G[0][j] .. G[m-1][j].  Each lane owns one column and
// keeps its values in registers as order-preserving integer keys.
//
// Only the middle of the order is needed, so no full sort is done: the m keys
// are padded to a compile-time width P with equally many -inf and +inf keys
// (one more +inf when P-m is odd), which pins the median to positions P/2-1 (m
// odd) or P/2-1 and P/2 (m even) of the sorted order.  The two halves are sorted
// by bitonic networks; one half-cleaner step min/max(a_i, b_{P/2-1-i}) then
// separates the P/2 smallest from the P/2 largest keys, and the two middle
// elements are the maximum of the former and the minimum of the latter.
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

// Ascending bitonic sort of v[0..H), fully unrolled (H is a power of two).
template <int H>
__device__ inline void sort_regs(int (&v)[H]) {
#pragma unroll
  for (int k = 2; k <= H; k <<= 1) {
#pragma unroll
    for (int s = k >> 1; s > 0; s >>= 1) {
#pragma unroll
      for (int i = 0; i < H; ++i) {
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
}

template <int P>
__global__ __launch_bounds__(kThreads) void median_kernel(const float* __restrict__ G, int m, long long d,
                                                          long long ldg, float* __restrict__ out) {
  constexpr int H = P / 2;
  const long long stride = (long long)gridDim.x * kThreads;
  const int f = (P - m) / 2;  // -inf keys in front; the rest of the padding is +inf keys behind
  for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < d; j += stride) {
    int a[H], b[H];
    // All P loads are issued back to back without branches: slot i reads row
    // min(i, m-1); the slots beyond m re-read the last row (cached) and are
    // overwritten by padding keys.  The address is kept as a per-lane pointer that
    // is stepped row by row (the empty asm keeps it in vector registers; a table
    // of P wave-uniform row addresses would not fit the scalar register file).
    const float* p = G + j;
    float val[P];
#pragma unroll
    for (int i = 0; i < P; ++i) {
      val[i] = *p;
      p += (i + 1 < m) ? ldg : 0;
      asm volatile("" : "+v"(p));
    }
#pragma unroll
    for (int i = 0; i < P; ++i) {
      // padding: the first f padding slots sort below everything, the rest above
      const int key = (i < m) ? float_key(val[i]) : (i - m < f ? INT_MIN : INT_MAX);
      if (i < H) a[i] = key; else b[i - H] = key;
    }
    sort_regs<H>(a);
    sort_regs<H>(b);
    int lo = INT_MIN, hi = INT_MAX;
#pragma unroll
    for (int i = 0; i < H; ++i) {
      const int x = a[i], y = b[H - 1 - i];
      const int mn = x < y ? x : y, mx = x < y ? y : x;
      lo = lo > mn ? lo : mn;
      hi = hi < mx ? hi : mx;
    }
    const float fa = key_float(lo), fb = key_float(hi);
    out[j] = (m & 1) ? fa : (float)(0.5 * ((double)fa + (double)fb));
  }
}

template <int P>
hipError_t launch_p(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream) {
  long long want = (d + kThreads - 1) / kThreads;
  int grid = (int)(want < 1 ? 1 : (want > 256 * 32 ? 256 * 32 : want));
  hipLaunchKernelGGL(median_kernel<P>, dim3(grid), dim3(kThreads), 0, stream, G, m, d, ldg, out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_median(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream) {
  if (m <= 2) return launch_p<2>(G, ldg, m, d, out, stream);
  if (m <= 4) return launch_p<4>(G, ldg, m, d, out, stream);
  if (m <= 8) return launch_p<8>(G, ldg, m, d, out, stream);
  if (m <= 16) return launch_p<16>(G, ldg, m, d, out, stream);
  if (m <= 32) return launch_p<32>(G, ldg, m, d, out, stream);
  if (m <= 64) return launch_p<64>(G, ldg, m, d, out, stream);
  return launch_p<128>(G, ldg, m, d, out, stream);
}

}  // namespace zeno
