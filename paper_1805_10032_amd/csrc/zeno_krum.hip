// Krum_b (Definition 5): the candidate with the smallest sum of squared distances to
// its m-b-2 nearest neighbours.  The O(d m^2) part is the Gram matrix S = G G^T, taken
// in one pass over G on the bf16 matrix cores at float32 accuracy: every float is split
// into three bf16 pieces x = h + m + l (round to nearest each, |m| <= 2^-8 |x|,
// |l| <= 2^-17 |x|) and the six piece products down to 2^-17 of the leading one
// (hh, hm, mh, mm, hl, lh) are accumulated in float32 (v_mfma_f32_32x32x16_bf16); what is
// dropped (ml, lm, ll and the split's remainder) is about 2^-24 of |x||y| per product,
// the size of one float32 rounding.  Six of these instructions cover 16
// columns in 192 cycles where the fp32 instruction (v_mfma_f32_32x32x2_f32) needs 512.
// The squared distances follow as S_ii + S_jj - 2 S_ij.
//
// That difference cancels when two rows are much closer to each other than to the origin
// (the honest workers' gradients late in training): its error is about 1e-7 of
// ||G_i||^2 + ||G_j||^2.  When a distance that enters a score is below 1e-3 of that scale
// (and the two rows are not bit-identical, whose distance is exactly 0), the whole
// computation is repeated on the rows minus the row that the first pass chose: distances do
// not change under a common shift, and the rows of the cluster around the chosen row then
// have norms of the size of their distances.  The second pass is decided on the device (a
// flag in the workspace) and its kernels return at once when it is not needed.
//
// krum_gram_kernel<RB>: the m <= 32 RB rows are cut into RB row blocks.  A wave owns a
// contiguous range of 64-column chunks; per chunk it loads the RB tiles of 32 rows x 64
// columns with coalesced 128-bit loads (rows at or beyond m read row m-1 and are
// zeroed), passes each through its wave-private XOR-swizzled LDS tile to reach operand
// order, and accumulates the RB(RB+1)/2 block products S_ab += T_a T_b^T, a <= b.  The
// four waves of a workgroup add their accumulators through LDS in a fixed tree and
// write one partial Gram per workgroup; krum_reduce_kernel sums the partials in
// float64 (fixed order), krum_score_kernel forms the score of one row per workgroup,
// krum_argmin_kernel picks the winner, krum_copy_kernel copies the winning row.
#include "zeno_layer_impl.h"

namespace zeno {

namespace {

constexpr int kGramWaves = 4;

typedef float f32x8 __attribute__((ext_vector_type(8)));

// Three-way split of eight floats into bf16 pieces, x = h + m + l + (at most 2^-25 |x|):
// h = bf16(x), m = bf16(x - h), l = bf16(x - h - m), round to nearest even each time;
// both subtractions are exact.
__device__ inline void split3(const f32x4& v0, const f32x4& v1, bf16x8& h, bf16x8& m, bf16x8& l) {
  const f32x8 x = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
  h = __builtin_convertvector(x, bf16x8);
  const f32x8 r1 = x - __builtin_convertvector(h, f32x8);
  m = __builtin_convertvector(r1, bf16x8);
  const f32x8 r2 = r1 - __builtin_convertvector(m, f32x8);
  l = __builtin_convertvector(r2, bf16x8);
}

// CENTER: second pass; runs only if *run_flag != 0 and subtracts row *center from every row.
template <int RB, bool CENTER>
__global__ __launch_bounds__(64 * kGramWaves, RB == 1 ? 3 : RB == 2 ? 2 : 1) void krum_gram_kernel(const float* __restrict__ G, long long ldg,
                                                                    int m, long long d, float* __restrict__ partial,
                                                                    const int32_t* __restrict__ center,
                                                                    const int32_t* __restrict__ run_flag) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  if (CENTER && *run_flag == 0) return;   // uniform over the launch
  const float* __restrict__ crow = CENTER ? G + (long long)(*center) * ldg : G;
  constexpr int PAIRS = RB * (RB + 1) / 2;
  constexpr int TILE_BYTES = 32 * 64 * 4;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned char* st = lds + wave * (RB * TILE_BYTES);
  const int rsub = lane >> 4, kq = (lane & 15) << 2;
  const int n = lane & 31, h = lane >> 5;

  f32x16 acc[PAIRS];
#pragma unroll
  for (int p = 0; p < PAIRS; ++p)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[p][j] = 0.f;

  // balanced contiguous share of the 64-column chunks for every wave of the launch
  const long long n_chunks = (d + 63) / 64;
  const long long w_global = (long long)blockIdx.x * kGramWaves + wave;
  const long long w_total = (long long)gridDim.x * kGramWaves;
  const long long c_begin = n_chunks * w_global / w_total, c_end = n_chunks * (w_global + 1) / w_total;

  // tile loads of chunk c into registers (rows at or beyond m read row m-1 and are zeroed)
  auto load_chunk = [&](f32x4 (&u)[RB][8], long long c) __attribute__((always_inline)) {
    const long long k0 = c * 64;
    const bool k_full = k0 + 64 <= d;  // wave-uniform
    f32x4 cv = {0.f, 0.f, 0.f, 0.f};
    if (CENTER) {
      if (k_full) cv = *reinterpret_cast<const f32x4_a4*>(crow + k0 + kq);
      else cv = load4_masked(crow + k0, kq, (int)(d - k0), true);
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = 32 * rb + 4 * j + rsub;
        const int rc = row < m ? row : m - 1;
        const float* p = G + (long long)rc * ldg + k0;
        f32x4 v;
        if (k_full) {
          v = load_stream4(p + kq);
        } else {
          v = load4_masked(p, kq, (int)(d - k0), true);
        }
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        u[rb][j] = row < m ? (CENTER ? v - cv : v) : zero;
      }
    }
  };
  // stage the tiles and accumulate the block products of one chunk
  auto products = [&](const f32x4 (&u)[RB][8]) __attribute__((always_inline)) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) stage_tile<false>(u[rb], st + rb * TILE_BYTES, lane);
    // operand fragments: per 16-column step s, lane (n, h) reads row n, columns
    // 16 s + 8 h .. + 7 of each tile and splits them into three bf16 pieces
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 fh[RB], fm[RB], fl[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const unsigned char* row = st + rb * TILE_BYTES + n * 256;
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(row + ((((4 * s + 2 * h) ^ n) & 15) << 4));
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(row + ((((4 * s + 2 * h + 1) ^ n) & 15) << 4));
        split3(v0, v1, fh[rb], fm[rb], fl[rb]);
      }
      int p = 0;
#pragma unroll
      for (int a = 0; a < RB; ++a)
#pragma unroll
        for (int b = a; b < RB; ++b, ++p) {
          const bf16x8 ah = fh[a], am = fm[a], al = fl[a], bh = fh[b], bm = fm[b], bl = fl[b];
          acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc[p], 0, 0, 0);
          acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc[p], 0, 0, 0);
          acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bm, acc[p], 0, 0, 0);
          acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh, acc[p], 0, 0, 0);
          acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bm, acc[p], 0, 0, 0);
          acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[p], 0, 0, 0);
        }
    }
  };

  if (RB <= 3) {
    // one chunk ahead in registers: the loads of chunk c+1 fly while chunk c is multiplied
    if (c_begin < c_end) {
      f32x4 u0[RB][8], u1[RB][8];
      load_chunk(u0, c_begin);
      long long c = c_begin;
      for (; c + 2 < c_end; c += 2) {
        load_chunk(u1, c + 1);
        products(u0);
        load_chunk(u0, c + 2);
        products(u1);
      }
      products(u0);
      if (c + 1 < c_end) {
        load_chunk(u1, c + 1);
        products(u1);
      }
    }
  } else {
    for (long long c = c_begin; c < c_end; ++c) {
      f32x4 u[RB][8];
      load_chunk(u, c);
      products(u);
    }
  }

  // sum the four waves' accumulators in a fixed tree, (0+2)+(1+3), through LDS
  float* red = reinterpret_cast<float*>(lds);
  for (int step = kGramWaves / 2; step >= 1; step >>= 1) {
    __syncthreads();
    if (wave >= step && wave < 2 * step) {
#pragma unroll
      for (int p = 0; p < PAIRS; ++p)
#pragma unroll
        for (int j = 0; j < 16; ++j) red[(((wave - step) * PAIRS + p) * 16 + j) * 64 + lane] = acc[p][j];
    }
    __syncthreads();
    if (wave < step) {
#pragma unroll
      for (int p = 0; p < PAIRS; ++p)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[p][j] += red[((wave * PAIRS + p) * 16 + j) * 64 + lane];
    }
  }
  if (wave == 0) {
    // accumulator element j of lane (n, h): row 8 (j/4) + 4 h + j%4 of block a, column n of block b
    float* out = partial + (long long)blockIdx.x * PAIRS * 1024;
#pragma unroll
    for (int p = 0; p < PAIRS; ++p)
#pragma unroll
      for (int j = 0; j < 16; ++j) out[p * 1024 + (8 * (j >> 2) + 4 * h + (j & 3)) * 32 + n] = acc[p][j];
  }
}

// Sum of the per-workgroup partial Grams in float64, in workgroup order: one thread per entry.
// pass 0 clears the flag that asks for the second pass; pass 1 runs only if it is set.
__global__ __launch_bounds__(256) void krum_reduce_kernel(const float* __restrict__ partial, int n_partials,
                                                          int entries, double* __restrict__ gram, int pass,
                                                          int32_t* __restrict__ flag) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (pass == 1 && *flag == 0) return;
  if (pass == 0 && e == 0) *flag = 0;   // (set, if at all, by the score kernel that follows)
  if (e >= entries) return;
  double t = 0.0;
  int w = 0;
  for (; w + 8 <= n_partials; w += 8) {   // eight loads in flight, added in workgroup order
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = partial[(long long)(w + q) * entries + e];
#pragma unroll
    for (int q = 0; q < 8; ++q) t += (double)v[q];
  }
  for (; w < n_partials; ++w) t += (double)partial[(long long)w * entries + e];
  gram[e] = t;
}

// Krum score of row i = blockIdx.x: squared distances to the other rows from the summed Gram
// blocks, ranked by counting (ties to the lower index), the m-b-2 smallest summed in
// ascending order.
__global__ __launch_bounds__(128) void krum_score_kernel(const double* __restrict__ gram, int rb, int m, int b,
                                                         double* __restrict__ score64, float* __restrict__ scores_out,
                                                         int pass, int32_t* __restrict__ flag) {
  __shared__ double dist[128];
  __shared__ double sorted[128];
  __shared__ int cancels[128];
  if (pass == 1 && *flag == 0) return;
  const int i = blockIdx.x, j = threadIdx.x;
  auto S = [&](int r, int c) {   // Gram entry (r, c), stored for block pairs a <= b only
    if (r > c) { const int t = r; r = c; c = t; }
    const int a = r >> 5, bb = c >> 5;
    const int p = a * rb - a * (a - 1) / 2 + (bb - a);
    return gram[p * 1024 + (r & 31) * 32 + (c & 31)];
  };
  if (j < m) {
    const double sii = S(i, i), sjj = S(j, j), sij = S(i, j);
    double dd = sii + sjj - 2.0 * sij;
    // the difference is rounding noise when it is far below the squares it is formed from, unless
    // the rows are bit-identical (all three entries equal, the distance exactly 0)
    cancels[j] = (j != i) && (dd < 1e-3 * (sii + sjj)) && !(sii == sjj && sii == sij);
    dd = dd < 0.0 ? 0.0 : dd;
    dd = (dd == dd) ? dd : __builtin_inf();      // a NaN/Inf row is infinitely far from every row: ranks stay a permutation
    dist[j] = (j == i) ? __builtin_inf() : dd;   // the row itself is never a neighbour
  }
  __syncthreads();
  if (j < m) {
    const double dj = dist[j];
    int rank = 0;
    for (int k = 0; k < m; ++k) {
      const double dk = dist[k];
      rank += (dk < dj) || (dk == dj && k < j);
    }
    sorted[rank] = dj;
    // a cancelling distance among the m-b-2 that enter the score: ask for the second pass
    if (pass == 0 && rank < m - b - 2 && cancels[j]) *flag = 1;
  }
  __syncthreads();
  if (j == 0) {
    double total = 0.0;
    for (int r = 0; r < m - b - 2; ++r) total += sorted[r];
    score64[i] = total;
    if (scores_out != nullptr) scores_out[i] = (float)total;
  }
}

// Winner: smallest score, ties to the lower index.
__global__ void krum_argmin_kernel(const double* __restrict__ score64, int m, int32_t* __restrict__ chosen, int pass,
                                   const int32_t* __restrict__ flag) {
  if (pass == 1 && *flag == 0) return;
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int best = 0;
    for (int i = 1; i < m; ++i)
      if (score64[i] < score64[best]) best = i;
    *chosen = best;
  }
}

__global__ __launch_bounds__(256) void krum_copy_kernel(const float* __restrict__ G, long long ldg, long long d,
                                                        const int32_t* __restrict__ chosen, float* __restrict__ out) {
  const float* row = G + (long long)(*chosen) * ldg;
  for (long long j = (long long)blockIdx.x * blockDim.x + threadIdx.x; j < d; j += (long long)gridDim.x * blockDim.x)
    out[j] = row[j];
}

template <int RB>
int gram_resident() {
  static const int cached = [] {
    int dev = 0, n_cu = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
      n_cu = 256;
    constexpr int lds = kGramWaves * RB * 32 * 64 * 4;
    if (lds > 48 * 1024)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&krum_gram_kernel<RB, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(&krum_gram_kernel<RB, false>),
                                                     64 * kGramWaves, lds) != hipSuccess || per_cu < 1)
      per_cu = 1;
    return n_cu * per_cu;
  }();
  return cached;
}

// workgroups of the Gram launch: as many as the chip holds at once
int gram_grid(int rb) {
  return rb == 1 ? gram_resident<1>() : rb == 2 ? gram_resident<2>() : rb == 3 ? gram_resident<3>() : gram_resident<4>();
}

template <int RB, bool CENTER>
hipError_t launch_gram(const float* G, long long ldg, int m, long long d, float* partial, int grid, const int32_t* center,
                       const int32_t* run_flag, hipStream_t stream) {
  constexpr int lds = kGramWaves * RB * 32 * 64 * 4;
  static const hipError_t attr_err =
      lds > 48 * 1024 ? hipFuncSetAttribute(reinterpret_cast<const void*>(&krum_gram_kernel<RB, CENTER>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds)
                      : hipSuccess;
  if (attr_err != hipSuccess) return attr_err;
  hipLaunchKernelGGL((krum_gram_kernel<RB, CENTER>), dim3(grid), dim3(64 * kGramWaves), lds, stream, G, ldg, m, d, partial,
                     center, run_flag);
  return hipGetLastError();
}

template <bool CENTER>
hipError_t launch_gram_rb(int rb, const float* G, long long ldg, int m, long long d, float* partial, int grid,
                          const int32_t* center, const int32_t* run_flag, hipStream_t stream) {
  if (rb == 1) return launch_gram<1, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  if (rb == 2) return launch_gram<2, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  if (rb == 3) return launch_gram<3, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  return launch_gram<4, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
}

}  // namespace

size_t krum_workspace_bytes(int m) {
  const int rb = (m + 31) / 32;
  const size_t entries = (size_t)(rb * (rb + 1) / 2) * 1024;
  return align_up((size_t)gram_grid(rb) * entries * sizeof(float), 256) + align_up(entries * sizeof(double), 256) +
         align_up(128 * sizeof(double), 256) + 256;   // partial Grams, summed Gram, scores, second-pass flag
}

hipError_t launch_krum(const float* G, long long ldg, int m, long long d, int b, float* out, int32_t* chosen,
                       float* scores_out, void* workspace, hipStream_t stream) {
  const int rb = (m + 31) / 32;
  const int grid = gram_grid(rb);
  float* partial = reinterpret_cast<float*>(workspace);
  const int entries = (rb * (rb + 1) / 2) * 1024;
  double* gram = reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(workspace) +
                                           align_up((size_t)grid * entries * sizeof(float), 256));
  double* score64 = gram + align_up((size_t)entries * sizeof(double), 256) / sizeof(double);
  int32_t* flag = reinterpret_cast<int32_t*>(score64 + align_up(128 * sizeof(double), 256) / sizeof(double));
  // pass 0 on the rows as they are; pass 1, only if pass 0 found a cancelling distance (decided on the
  // device: its kernels return at once otherwise), on the rows minus the row pass 0 chose
  for (int pass = 0; pass < 2; ++pass) {
    hipError_t e = pass == 0 ? launch_gram_rb<false>(rb, G, ldg, m, d, partial, grid, nullptr, nullptr, stream)
                             : launch_gram_rb<true>(rb, G, ldg, m, d, partial, grid, chosen, flag, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(krum_reduce_kernel, dim3((entries + 255) / 256), dim3(256), 0, stream, partial, grid, entries, gram,
                       pass, flag);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(krum_score_kernel, dim3(m), dim3(128), 0, stream, gram, rb, m, b, score64, scores_out, pass, flag);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(krum_argmin_kernel, dim3(1), dim3(64), 0, stream, score64, m, chosen, pass, flag);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  long long want = (d + 255) / 256;
  const int cgrid = (int)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
  hipLaunchKernelGGL(krum_copy_kernel, dim3(cgrid), dim3(256), 0, stream, G, ldg, d, chosen, out);
  return hipGetLastError();
}

}  // namespace zeno
