// Marginal median (Definition 4): for every coordinate j the one-dimensional
// median of the m values G[0][j] .. G[m-1][j].  Each lane owns one column (four
// adjacent ones up to m = 32, read with one 128-bit load per row) and keeps its
// values in registers as order-preserving integer keys.
//
// Only the middle of the order is needed, so no full sort is done: the m keys
// are padded to a power of two P with equally many -inf and +inf keys (one more
// +inf when P-m is odd), which pins the median to positions P/2-1 (m odd) or
// P/2-1 and P/2 (m even) of the sorted order.  The two halves are sorted by
// Batcher's odd-even merge sort (every compare-exchange ascending); one
// half-cleaner step min/max(a_i, b_{P/2-1-i}) then separates the P/2 smallest
// from the P/2 largest keys, and the two middle elements are the maximum of the
// former and the minimum of the latter.
//
// Most of the padding sits at positions fixed at compile time: the kernel is
// instantiated for Q real slots (m rounded up to a multiple of 4, of 8 above
// 64), the lowest (P-Q)/2 positions of the first half hold the constant -inf key and the
// highest (P-Q)/2 of the second half the constant +inf key.  An ascending
// compare-exchange never moves those, so after unrolling the compiler deletes
// every compare-exchange that touches one: the network that runs is the one for
// Q keys, not for P.  The Q-m slots left over are padded at run time.
#include <limits.h>
#include <stdint.h>

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

// Ascending odd-even merge sort of v[0..H), fully unrolled (H is a power of two).
template <int H>
__device__ inline void sort_regs(int (&v)[H]) {
#pragma unroll
  for (int p = 1; p < H; p <<= 1) {
#pragma unroll
    for (int k = p; k >= 1; k >>= 1) {
#pragma unroll
      for (int j = k % p; j + k < H; j += 2 * k) {
#pragma unroll
        for (int i = 0; i < k; ++i) {
          const int lo = i + j, hi = i + j + k;
          if (hi < H && lo / (2 * p) == hi / (2 * p)) {
            const int a = v[lo], c = v[hi];
            v[lo] = a < c ? a : c;
            v[hi] = a < c ? c : a;
          }
        }
      }
    }
  }
}

template <int P, int Q, int VEC, bool NT>
__global__ __launch_bounds__(kThreads) void median_kernel(const float* __restrict__ G, int m, long long d,
                                                          long long ldg, float* __restrict__ out) {
  typedef float vf __attribute__((ext_vector_type(VEC)));
  constexpr int H = P / 2;
  constexpr int C = (P - Q) / 2;  // constant keys per half
  static_assert(P == Q || (Q % 4 == 0 && Q < P && Q > P / 2), "Q real slots, more than half of P");
  const long long stride = (long long)gridDim.x * kThreads;
  const long long n_vec = d / VEC;  // the launcher sends the d % VEC columns left over to the VEC = 1 kernel
  const int f = (Q - m) / 2;        // run-time -inf keys; the rest of the run-time padding is +inf keys
  for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < n_vec; j += stride) {
    // Each lane owns VEC adjacent columns and reads them with one load per row.
    // All Q loads are issued back to back without branches: slot i reads row
    // min(i, m-1); the slots beyond m re-read the last row (cached) and are
    // overwritten by padding keys.  The address is kept as a per-lane pointer that
    // is stepped row by row (the empty asm keeps it in vector registers; a table
    // of wave-uniform row addresses would not fit the scalar register file).
    const float* p = G + j * VEC;
    vf val[Q];
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      if constexpr (NT) {
        val[i] = __builtin_nontemporal_load(reinterpret_cast<const vf*>(p));
      } else {
        val[i] = *reinterpret_cast<const vf*>(p);
      }
      p += (i + 1 < m) ? ldg : 0;
      asm volatile("" : "+v"(p));
    }
    vf res;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      int a[H], b[H];
      auto slot_key = [&](int i) {
        // run-time padding: the first f padding slots sort below everything, the rest above
        return (i < m) ? float_key(val[i][v]) : (i - m < f ? INT_MIN : INT_MAX);
      };
#pragma unroll
      for (int i = 0; i < C; ++i) a[i] = INT_MIN;
#pragma unroll
      for (int i = 0; i < H - C; ++i) a[C + i] = slot_key(i);
#pragma unroll
      for (int i = 0; i < C; ++i) b[H - 1 - i] = INT_MAX;
#pragma unroll
      for (int i = H - C; i < Q; ++i) b[i - (H - C)] = slot_key(i);
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
      const float r = (m & 1) ? fa : (float)(0.5 * ((double)fa + (double)fb));
      res[v] = r;
    }
    *reinterpret_cast<vf*>(out + j * VEC) = res;
  }
}

// Rows that start on cache-line boundaries are read with streaming (nontemporal)
// loads when m is small: every line is used once by one wave, and at small m the
// kernel is bound by the loads alone.  Rows that straddle lines keep ordinary loads,
// which let the neighbouring wave find the shared line in cache.
template <int P, int Q, int VEC>
hipError_t launch_vec(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream) {
  long long want = (d / VEC + kThreads - 1) / kThreads;
  int grid = (int)(want < 1 ? 1 : (want > 256 * 32 ? 256 * 32 : want));
  if constexpr (Q <= 48) {
    if (ldg % 32 == 0 && reinterpret_cast<uintptr_t>(G) % 128 == 0) {
      hipLaunchKernelGGL((median_kernel<P, Q, VEC, true>), dim3(grid), dim3(kThreads), 0, stream, G, m, d, ldg, out);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((median_kernel<P, Q, VEC, false>), dim3(grid), dim3(kThreads), 0, stream, G, m, d, ldg, out);
  return hipGetLastError();
}

// Lanes take kVec<Q> columns each when every row and the output are aligned for
// that load width; the d % VEC columns left over go to the one-column kernel.
template <int Q>
constexpr int kVecFor = Q <= 32 ? 4 : 1;

template <int P, int Q>
hipError_t launch_pq(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream) {
  constexpr int VEC = kVecFor<Q>;
  if constexpr (VEC > 1) {
    const bool aligned = ldg % VEC == 0 && reinterpret_cast<uintptr_t>(G) % (4 * VEC) == 0 &&
                         reinterpret_cast<uintptr_t>(out) % (4 * VEC) == 0;
    if (aligned && d >= VEC) {
      hipError_t e = launch_vec<P, Q, VEC>(G, ldg, m, d, out, stream);
      const long long done = d / VEC * VEC;
      if (e != hipSuccess || done == d) return e;
      return launch_vec<P, Q, 1>(G + done, ldg, m, d - done, out + done, stream);
    }
  }
  return launch_vec<P, Q, 1>(G, ldg, m, d, out, stream);
}

// Q = m rounded up to a multiple of kStep inside (P/2, P]: 4 up to P = 64, 8 for P = 128.
template <int P, int Q>
hipError_t launch_q(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream) {
  constexpr int kStep = P > 64 ? 8 : 4;
  if constexpr (Q >= P) {
    return launch_pq<P, P>(G, ldg, m, d, out, stream);
  } else {
    if (m <= Q) return launch_pq<P, Q>(G, ldg, m, d, out, stream);
    return launch_q<P, Q + kStep>(G, ldg, m, d, out, stream);
  }
}

template <int P>
hipError_t launch_p(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream) {
  if constexpr (P >= 16) {
    return launch_q<P, P / 2 + (P > 64 ? 8 : 4)>(G, ldg, m, d, out, stream);
  } else {
    return launch_pq<P, P>(G, ldg, m, d, out, stream);
  }
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
