// Selection of the m-b highest scores and the average of the selected rows
// (Definition 3, Zeno_b), and the Mean baseline (Section 6.1.1) as the b = 0
// case without scores.  One streaming pass over the selected rows of G.
#include "zeno_internal.h"

namespace zeno {

namespace {

constexpr int kThreads = 256;

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

// Results leave the workgroup in large contiguous bursts: a workgroup averages
// n_blocks consecutive column blocks of kBlockVec float4 columns each, parks the
// results in LDS and then writes the whole run (up to 144 KB) at once.  Measured
// on MI355X, output stores that trickle out between the row loads cost about a
// fifth of the read bandwidth although they are 1/(n_sel+1) of the bytes; written
// in bursts (and marked write-through, so they do not linger as dirty lines) they
// cost a few percent.
constexpr int kVec = 4;                      // float4 columns per thread and block
constexpr int kBlockVec = kThreads * kVec;   // float4 columns per block (16 KB of output)
// rows whose loads are in flight together (x kVec loads each); the variant that
// looks its rows up in the selected list keeps more in flight to cover the lookup
constexpr int kRowsAll = 2, kRowsSel = 4;
constexpr int kMaxBlocks = 9;                // blocks per burst: 9 x 16 KB of LDS

__device__ inline void store_burst(float* p, const f32x4& v) {
  // 16-byte store, write-through to memory (system-coherent scope bit): the line is
  // not kept dirty in the L2, which the streaming row loads would have to displace
  // (s_nop: a store wider than 64 bits reads its data registers for two more cycles,
  // and the compiler does not add the wait states it gives its own stores to assembly)
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}

// The SGD step of Algorithm 1 (server side), x_next = x - gamma * aggregate, from the
// float64 average before it is rounded: one rounding to fp32 in all.  Contraction is
// off so that the product and the difference are rounded separately, as written.
__device__ inline float sgd_step(float x, double gamma, double avg) {
#pragma clang fp contract(off)
  const double step = gamma * avg;
  return (float)((double)x - step);
}

// UPDATE: also (or only, out == nullptr) write x_next = x - gamma * average; x_next may
// be x itself (every column is read and written by one thread).
template <bool ALL, bool UPDATE>
__global__ __launch_bounds__(kThreads) void masked_average_kernel(const float* __restrict__ G,
                                                                  const float* __restrict__ scores, int m,
                                                                  long long d, long long ldg, int b, int n_blocks,
                                                                  float* __restrict__ out,
                                                                  int32_t* __restrict__ selected, float gamma,
                                                                  const float* x, float* x_next) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  // [selected row list][burst buffer]; the selection's scratch (keys, flags) lies
  // in the burst buffer, which is not used before the selection is over
  int* sel_list = reinterpret_cast<int*>(lds_raw);
  f32x4* burst = reinterpret_cast<f32x4*>(lds_raw + ZENO_MAX_CANDIDATES * sizeof(int));
  const int n_sel = ALL ? m : m - b;
  if (!ALL) {
    float* key = reinterpret_cast<float*>(burst);
    int* flag = reinterpret_cast<int*>(key + ZENO_MAX_CANDIDATES);
    select_rows(scores, m, n_sel, key, flag, sel_list, blockIdx.x == 0 ? selected : nullptr);
  }

  const double n = (double)n_sel;
  // second burst buffer (new parameters) behind the first (average) when both are written
  const int xoff = (UPDATE && out != nullptr) ? n_blocks * kBlockVec : 0;
  const long long n_vec = d / 4;
  // balanced contiguous share of the column blocks, worked through in bursts of n_blocks
  const long long blocks_total = (n_vec + kBlockVec - 1) / kBlockVec;
  const long long blk_begin = blocks_total * blockIdx.x / gridDim.x;
  const long long blk_end = blocks_total * (blockIdx.x + 1) / gridDim.x;
  for (long long g = blk_begin; g < blk_end; g += n_blocks) {
    const int nb = (int)(blk_end - g < n_blocks ? blk_end - g : n_blocks);
    for (int i = 0; i < nb; ++i) {
      const long long c0 = (g + i) * kBlockVec + threadIdx.x;
      double acc[kVec][4];
#pragma unroll
      for (int v = 0; v < kVec; ++v)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[v][e] = 0.0;
      // columns beyond the end re-read the last full column (in bounds) and are not written
      long long col[kVec];
#pragma unroll
      for (int v = 0; v < kVec; ++v) {
        const long long c = c0 + v * kThreads;
        col[v] = (c < n_vec ? c : n_vec - 1) * 4;
      }
      f32x4 xv[kVec];
      if (UPDATE) {
#pragma unroll
        for (int v = 0; v < kVec; ++v) xv[v] = *reinterpret_cast<const f32x4_a4*>(x + col[v]);
      }
      constexpr int RB = ALL ? kRowsAll : kRowsSel;
      int s = 0;
      // the list entries of the NEXT batch are fetched while this batch's loads are
      // in flight (entries past the end repeat the last one and are never used)
      int rows[RB];
#pragma unroll
      for (int t = 0; t < RB; ++t) rows[t] = ALL ? t : sel_list[t < n_sel ? t : n_sel - 1];
      for (; s + RB <= n_sel; s += RB) {
        f32x4 x[RB][kVec];
#pragma unroll
        for (int t = 0; t < RB; ++t) {
          const float* rp = G + (long long)rows[t] * ldg;
#pragma unroll
          for (int v = 0; v < kVec; ++v) x[t][v] = load_stream4(rp + col[v]);
        }
        // keep the whole batch of loads in flight: without the fences the scheduler
        // interleaves loads and additions to save registers and waits after every few loads
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < RB; ++t) {
          const int nx = s + RB + t;
          rows[t] = ALL ? nx : sel_list[nx < n_sel ? nx : n_sel - 1];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < RB; ++t)
#pragma unroll
          for (int v = 0; v < kVec; ++v)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[v][e] += (double)x[t][v][e];
      }
      for (; s < n_sel; ++s) {
        const long long row = ALL ? s : sel_list[s];
        f32x4 x[kVec];
#pragma unroll
        for (int v = 0; v < kVec; ++v) x[v] = load_stream4(G + row * ldg + col[v]);
#pragma unroll
        for (int v = 0; v < kVec; ++v)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[v][e] += (double)x[v][e];
      }
#pragma unroll
      for (int v = 0; v < kVec; ++v) {
        f32x4 r, xn;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const double avg = acc[v][e] / n;
          r[e] = (float)avg;
          if (UPDATE) xn[e] = sgd_step(xv[v][e], (double)gamma, avg);
        }
        const int slot = i * kBlockVec + v * kThreads + threadIdx.x;
        if (!UPDATE || out != nullptr) burst[slot] = r;
        if (UPDATE) burst[xoff + slot] = xn;
      }
    }
    __syncthreads();
    const long long g0 = g * kBlockVec;
    const long long left = n_vec - g0;
    const int n_out = (int)(left < (long long)nb * kBlockVec ? left : (long long)nb * kBlockVec);
    if (!UPDATE || out != nullptr)
      for (int j = threadIdx.x; j < n_out; j += kThreads) store_burst(out + (g0 + j) * 4, burst[j]);
    if (UPDATE)
      for (int j = threadIdx.x; j < n_out; j += kThreads)
        store_burst(x_next + (g0 + j) * 4, burst[xoff + j]);
    __syncthreads();
  }
  // d mod 4 trailing columns
  if (blockIdx.x == 0) {
    for (long long j = n_vec * 4 + threadIdx.x; j < d; j += kThreads) {
      double a = 0.0;
      for (int s = 0; s < n_sel; ++s) {
        const long long row = ALL ? s : sel_list[s];
        a += (double)G[row * ldg + j];
      }
      if (!UPDATE || out != nullptr) out[j] = (float)(a / n);
      if (UPDATE) x_next[j] = sgd_step(x[j], (double)gamma, a / n);
    }
  }
}

}  // namespace

hipError_t launch_masked_average(const float* G, long long ldg, const float* scores, int m, long long d, int b,
                                 float* out, int32_t* selected, hipStream_t stream, float gamma, const float* x,
                                 float* x_next) {
  const bool update = x_next != nullptr;
  const int n_bufs = (update && out != nullptr) ? 2 : 1;   // burst buffers: the average, the new parameters
  const int max_blocks = kMaxBlocks / n_bufs;
  const long long n_vec = d / 4;
  // burst length: as long as LDS allows while at least ~512 workgroups' worth of groups remain
  long long nb = n_vec / ((long long)kBlockVec * 512);
  const int n_blocks = (int)(nb < 1 ? 1 : (nb > max_blocks ? max_blocks : nb));
  const size_t lds = ZENO_MAX_CANDIDATES * sizeof(int) + (size_t)n_bufs * n_blocks * kBlockVec * 16;
  // as many workgroups as the chip holds at once (LDS-limited), each with a balanced share of the blocks
  static const int n_cu = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
      v = 256;
    return v;
  }();
  int per_cu = (int)((160 * 1024) / (lds + 512));
  per_cu = per_cu < 1 ? 1 : (per_cu > 8 ? 8 : per_cu);
  const long long blocks_total = (n_vec + kBlockVec - 1) / kBlockVec;
  const long long resident = (long long)n_cu * per_cu;
  const int grid = (int)(blocks_total < 1 ? 1 : (blocks_total > resident ? resident : blocks_total));
  // once per process (initialisation of a local static is thread-safe)
  static const hipError_t attr_err = [] {
    const int lds_max = (int)(ZENO_MAX_CANDIDATES * sizeof(int) + (size_t)kMaxBlocks * kBlockVec * 16);
    const void* kernels[4] = {reinterpret_cast<const void*>(&masked_average_kernel<true, false>),
                              reinterpret_cast<const void*>(&masked_average_kernel<false, false>),
                              reinterpret_cast<const void*>(&masked_average_kernel<true, true>),
                              reinterpret_cast<const void*>(&masked_average_kernel<false, true>)};
    for (const void* k : kernels) {
      hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }();
  if (attr_err != hipSuccess) return attr_err;
  const bool all = scores == nullptr;
  const int bb = all ? 0 : b;
#define ZENO_LAUNCH_AVG(ALLV, UPD)                                                                                  \
  hipLaunchKernelGGL((masked_average_kernel<ALLV, UPD>), dim3(grid), dim3(kThreads), lds, stream, G, scores, m, d, \
                     ldg, bb, n_blocks, out, selected, gamma, x, x_next)
  if (all && !update) ZENO_LAUNCH_AVG(true, false);
  else if (all) ZENO_LAUNCH_AVG(true, true);
  else if (!update) ZENO_LAUNCH_AVG(false, false);
  else ZENO_LAUNCH_AVG(false, true);
#undef ZENO_LAUNCH_AVG
  return hipGetLastError();
}

}  // namespace zeno
