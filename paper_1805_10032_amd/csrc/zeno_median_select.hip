// Marginal median (Definition 4) for more rows than the register-resident sorting
// networks of zeno_median.hip hold: 128 < m <= 1024.
//
// A workgroup of eight waves takes 32 adjacent columns at a time.  Their m x 32 values are
// read once (a wave's load instruction covers two rows x 128 contiguous bytes), turned into
// order-preserving integer keys and kept in LDS column by column.  Sixteen lanes share a
// column.  The lower median, the key of rank k = (m - 1) / 2, is then found bit by bit
// from the top: a bit stays set in the threshold T if no more than k keys lie below
// T with that bit set, which leaves T = the largest value with #{key < T} <= k, i.e.
// the key of rank k itself.  Every step is one pass of the sixteen lanes over their share
// of the column and a four-step shuffle sum.  For even m one more pass finds the key of
// rank k + 1 (T again if enough keys equal T, else the smallest key above T), and the
// result is the midpoint of the two, formed in float64 and rounded once, as in the
// kernels for m <= 128.  NaN entries sort above +inf.
//
// A lane reads its share of a column four keys at a time (128-bit LDS reads, rows 4 part + 64 i .. + 3), two
// such reads in flight, so a column holds m rounded up to a multiple of 128 keys; the rows beyond m hold the top
// key, which no threshold counts as below it.  The sixteen lanes that one phase of a 128-bit read serves are the
// lanes of one column and read 256 contiguous bytes: all 64 banks once.  The column stride is the padded length
// plus 32 words, which spreads the transposing writes of the fill over the banks.
// Measured (MI355X): m = 256 .. 1024 run at 0.75-0.9 TB/s of G, bound by the 32 counting passes (plain ALU), i.e.
// several times slower per byte than the sorting networks; m = 129 pays for its padding to 256 keys (0.5 TB/s).
#include <limits.h>
#include <stdint.h>

#include "zeno_internal.h"

namespace zeno {

namespace {

constexpr int kSelThreads = 512;
constexpr int kSelCols = 32;    // columns per tile
constexpr int kSelShare = 16;   // lanes per column

// float -> unsigned key whose unsigned order is -inf < ... < -0 < +0 < ... < +inf < NaN
__device__ inline unsigned sel_key(float f) {
  int k = __float_as_int(f);
  k ^= (k >> 31) & 0x7fffffff;
  k = (f != f) ? INT_MAX : k;
  return (unsigned)k ^ 0x80000000u;
}
__device__ inline float sel_float(unsigned u) {
  const int k = (int)(u ^ 0x80000000u);
  return __int_as_float(k ^ ((k >> 31) & 0x7fffffff));
}

__device__ inline int share_sum(int v) {
  v += __shfl_xor(v, 1, 64);
  v += __shfl_xor(v, 2, 64);
  v += __shfl_xor(v, 4, 64);
  v += __shfl_xor(v, 8, 64);
  return v;
}
__device__ inline unsigned share_min(unsigned v) {
  unsigned o = __shfl_xor(v, 1, 64);
  v = o < v ? o : v;
  o = __shfl_xor(v, 2, 64);
  v = o < v ? o : v;
  o = __shfl_xor(v, 4, 64);
  v = o < v ? o : v;
  o = __shfl_xor(v, 8, 64);
  return o < v ? o : v;
}

__global__ __launch_bounds__(kSelThreads) void median_select_kernel(const float* __restrict__ G, int m, long long d,
                                                                    long long ldg, int stride, float* __restrict__ out) {
  extern __shared__ unsigned keys[];   // [kSelCols][stride]
  const int tid = threadIdx.x;
  const long long n_tiles = (d + kSelCols - 1) / kSelCols;
  const int k = (m - 1) / 2;
  const int mp = stride - 32;          // rows per column in LDS, a multiple of 128
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  // the padding rows m .. mp-1 of every column: written once, the tiles only overwrite rows below m
  for (int i = tid; i < kSelCols * (mp - m); i += kSelThreads) keys[(i / (mp - m)) * stride + m + i % (mp - m)] = 0xffffffffu;
  for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const long long col0 = tile * kSelCols;
    {
      // fill: lane = column, sixteen rows per pass of the workgroup, eight passes in flight
      const int c = tid & (kSelCols - 1), r0 = tid >> 5;
      const bool col_ok = col0 + c < d;
      const float* p = G + (col_ok ? col0 + c : 0);
      int r = r0;
      constexpr int RPP = kSelThreads / kSelCols;   // rows per pass
      for (; r + 7 * RPP < m; r += 8 * RPP) {
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = p[(long long)(r + RPP * q) * ldg];
#pragma unroll
        for (int q = 0; q < 8; ++q) keys[c * stride + r + RPP * q] = sel_key(v[q]);
      }
      for (; r < m; r += RPP) keys[c * stride + r] = sel_key(p[(long long)r * ldg]);
    }
    __syncthreads();
    {
      const int c = tid / kSelShare, part = tid & (kSelShare - 1);
      const u32x4* col = reinterpret_cast<const u32x4*>(keys + c * stride) + part;   // the lane's keys: col[kSelShare i]
      const int n_reads = mp / (4 * kSelShare);   // a multiple of 2
      unsigned T = 0u;
      for (int bit = 31; bit >= 0; --bit) {
        const unsigned cand = T | (1u << bit);
        int below = 0;
        for (int i = 0; i < n_reads; i += 2) {
          u32x4 v[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) v[q] = col[kSelShare * (i + q)];
#pragma unroll
          for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) below += v[q][e] < cand ? 1 : 0;
        }
        below = share_sum(below);
        T = below <= k ? cand : T;
      }
      float res = sel_float(T);
      if ((m & 1) == 0) {
        // rank k + 1: T again if more than k + 1 keys are <= T, else the smallest key above T (the padding keys
        // can only be counted or picked where T or that key is the top key itself)
        int le = 0;
        unsigned above = 0xffffffffu;
        for (int i = 0; i < n_reads; ++i) {
          const u32x4 v = col[kSelShare * i];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            le += v[e] <= T ? 1 : 0;
            above = (v[e] > T && v[e] < above) ? v[e] : above;
          }
        }
        le = share_sum(le);
        above = share_min(above);
        const unsigned U = le > k + 1 ? T : above;
        res = (float)(0.5 * ((double)res + (double)sel_float(U)));
      }
      if (part == 0 && col0 + c < d) out[col0 + c] = res;
    }
    __syncthreads();   // the keys are overwritten by the next tile
  }
}

}  // namespace

hipError_t launch_median_select(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream) {
  const int stride = (m + 127) / 128 * 128 + 32;
  const int lds_bytes = kSelCols * stride * (int)sizeof(unsigned);
  static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&median_select_kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, kSelCols * (1024 + 32) * (int)sizeof(unsigned));
  if (attr_err != hipSuccess) return attr_err;
  if (m > 1024) return hipErrorInvalidValue;   // the attribute above covers the stride of m = 1024
  int dev = 0, n_cu = 256;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    n_cu = 256;
  int per_cu = (160 * 1024) / lds_bytes;
  if (per_cu > 8) per_cu = 8;
  if (per_cu < 1) per_cu = 1;
  const long long n_tiles = (d + kSelCols - 1) / kSelCols;
  const long long want = (long long)n_cu * per_cu;
  const int grid = (int)(n_tiles < want ? n_tiles : want);
  hipLaunchKernelGGL(median_select_kernel, dim3(grid), dim3(kSelThreads), lds_bytes, stream, G, m, d, ldg, stride, out);
  return hipGetLastError();
}

}  // namespace zeno
