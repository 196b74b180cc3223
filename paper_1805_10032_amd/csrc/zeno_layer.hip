// Streaming layer kernel of the Stochastic Descendant Score (Definition 2).
//
// For one linear layer l and every source s of the launch (candidate rows G[s],
// s < m, and the current parameters x as source m) a workgroup owns BN = 32*NW
// output features and streams the corresponding rows of that source's weight
// block from HBM exactly once, K-chunk by K-chunk:
//
//   source m (pass at x):   Z0   = H0 W^T + b                 (pre-activations at x)
//   source s < m:           dZ_s = -gamma ( H_s U_s^T + D_s W^T + ub_s )
//
// where H_s are candidate s's input activations, U_s / ub_s its weight / bias
// block, and D_s = (H_s - H0) * (-1/gamma) the scaled change of the input
// activations (absent at the first layer, where H_s = H0 = the batch).  dZ_s is
// the change of the pre-activations caused by moving x to x - gamma u_s, so the
// perturbed parameters are never formed and f_r(x) - f_r(x - gamma u) is later
// obtained without subtracting two nearly equal losses.  ||u_s||^2 is
// accumulated from the same registers that feed the matrix cores.
//
// Matrix-core mapping (wave64): each wave owns 32 output features (columns of the
// 32x32 accumulator blocks) and all MB*32 sample rows.  The weight tile is
// loaded with fully coalesced 128-bit loads (4 rows x 256 B per instruction),
// converted, and passed through a wave-private LDS tile to reach the operand
// layout (lane = feature, 8 consecutive k); the activation operands are stored
// in global memory already in operand order ("tiled") and are shared by the
// waves of the workgroup through LDS.
#include "zeno_internal.h"

namespace zeno {

namespace {

template <bool BF16>
struct Tr;
template <>
struct Tr<true> {
  static constexpr int ESIZE = 2;
  static constexpr int CH_BYTES = 32 * 64 * 2;  // one 32-row block of a 64-wide K chunk, tiled operand
  static constexpr int STAGE_ROW = 64 * 2 + 16; // staged weight row: 64 bf16 + pad (conflict-free b128 reads)
};
template <>
struct Tr<false> {
  static constexpr int ESIZE = 4;
  static constexpr int CH_BYTES = 32 * 64 * 4;
  static constexpr int STAGE_ROW = 64 * 4 + 16;
};

// Element index of (row r, column k) inside a tiled activation operand of padded
// width Kp.  bf16: blocks of 32 rows x 16 k, lane = r%32 + 32*((k%16)/8), 8
// consecutive k per lane (the operand layout of the 32x32x16 bf16 matrix
// instruction).  fp32: blocks of 32 rows x 8 k, lane = r%32 + 32*((k%8)/4), the
// four values of a lane feed four consecutive 32x32x2 fp32 instructions.
template <bool BF16>
__host__ __device__ inline long long tiled_index(int r, int k, int Kp) {
  if (BF16) {
    return ((((long long)(r >> 5) * (Kp >> 4) + (k >> 4)) * 64 + (r & 31) + 32 * ((k & 15) >> 3)) << 3) + (k & 7);
  } else {
    return ((((long long)(r >> 5) * (Kp >> 3) + (k >> 3)) * 64 + (r & 31) + 32 * ((k & 7) >> 2)) << 2) + (k & 3);
  }
}

template <bool BF16>
__device__ inline void store_tiled(void* base, int r, int k, int Kp, float v) {
  const long long idx = tiled_index<BF16>(r, k, Kp);
  if (BF16) {
    reinterpret_cast<__bf16*>(base)[idx] = (__bf16)v;
  } else {
    reinterpret_cast<float*>(base)[idx] = v;
  }
}

// Output features a launch must cover: a hidden layer also writes the zero
// padding of the next layer's tiled operand (width rounded up to 64).
__host__ __device__ inline int cover_rows(int N, int last) { return last ? N : (N + 63) / 64 * 64; }

// NaN-propagating ReLU (fmaxf would swallow a NaN coming from a faulty row).
__device__ inline float relu_nan(float v) { return (v <= 0.0f) ? 0.0f : v; }

__device__ inline f32x4 load4_masked(const float* __restrict__ row, int k, int K, bool row_ok) {
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (row_ok) {
    if (k + 4 <= K) {
      const f4u t = *reinterpret_cast<const f4u*>(row + k);
      v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
      if (k < K) v[0] = row[k];
      if (k + 1 < K) v[1] = row[k + 1];
      if (k + 2 < K) v[2] = row[k + 2];
    }
  }
  return v;
}

// Load the wave's 32 x 64 weight tile: instruction j covers rows 4j..4j+3, 256
// contiguous bytes each.
__device__ inline void load_tile(f32x4 (&u)[8], const float* __restrict__ mat, int row0, int k0, int N, int K,
                                 int lane) {
  const int rsub = lane >> 4, k = k0 + ((lane & 15) << 2);
  if (row0 + 32 <= N && k0 + 64 <= K) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const f4u t = *reinterpret_cast<const f4u*>(mat + (long long)(row0 + 4 * j + rsub) * K + k);
      u[j][0] = t.x; u[j][1] = t.y; u[j][2] = t.z; u[j][3] = t.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row = row0 + 4 * j + rsub;
      u[j] = load4_masked(mat + (long long)row * K, k, K, row < N);
    }
  }
}

template <bool BF16>
__device__ inline void stage_tile(const f32x4 (&u)[8], unsigned char* st, int lane) {
  using T = Tr<BF16>;
  const int rsub = lane >> 4, kq = lane & 15;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    unsigned char* p = st + (4 * j + rsub) * T::STAGE_ROW;
    if (BF16) {
      const bf16x4 h = __builtin_convertvector(u[j], bf16x4);
      *reinterpret_cast<bf16x4*>(p + kq * 8) = h;
    } else {
      *reinterpret_cast<f32x4*>(p + kq * 16) = u[j];
    }
  }
}

template <bool BF16, bool DELTA, int MB, int NW>
__global__ __launch_bounds__(64 * NW) void layer_kernel(const LayerArgs a) {
  using T = Tr<BF16>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int NT = 64 * NW;
  constexpr int BN = 32 * NW;
  constexpr int A_BYTES = MB * T::CH_BYTES;
  constexpr int A_PIECES = A_BYTES / 16;
  constexpr int APT = (A_PIECES + NT - 1) / NT;
  constexpr int PIECES_PER_BLOCK = T::CH_BYTES / 16;
  constexpr int STAGE_BYTES = 32 * T::STAGE_ROW;
  constexpr int N_STAGE = DELTA ? 2 : 1;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  unsigned char* ldsA = lds;
  unsigned char* ldsD = lds + A_BYTES;
  unsigned char* stU = lds + A_BYTES * N_STAGE + wave * (STAGE_BYTES * N_STAGE);
  unsigned char* stW = stU + STAGE_BYTES;

  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2):
  // consecutive slots of one XCD walk through the feature tiles of one source,
  // so that a source's activations are fetched into a single L2.
  const int n_tiles = (cover_rows(a.N, a.last) + BN - 1) / BN;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int src_local = (slot / n_tiles) * 8 + xcd;
  const int nt = slot % n_tiles;
  if (src_local >= a.n_src) return;
  const int s = a.src_begin + src_local;
  const bool is_base = (s == a.m);
  const float* __restrict__ P = is_base ? a.x : a.G + (long long)s * a.d;
  const float* __restrict__ Umat = P + a.w_off;
  const float* __restrict__ Wmat = a.x + a.w_off;
  const int row0 = nt * BN + wave * 32;
  const int N = a.N, K = a.K;
  const int n_chunks = a.Kp >> 6;

  const unsigned char* Ag = reinterpret_cast<const unsigned char*>(a.A_base);
  if (!is_base && a.A_cand != nullptr) Ag = reinterpret_cast<const unsigned char*>(a.A_cand) + (long long)s * a.A_stride;
  const unsigned char* Dg = DELTA ? reinterpret_cast<const unsigned char*>(a.D_cand) + (long long)s * a.A_stride : nullptr;

  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[mb][j] = 0.f;

  const bool do_norm = (a.norm_partials != nullptr) && !is_base;
  double nrm = 0.0;

  f32x4 u[8], w[8];
  f32x4 pa[APT], pd[APT];

  auto load_A = [&](int c) {
#pragma unroll
    for (int i = 0; i < APT; ++i) {
      const int p = tid + i * NT;
      if (A_PIECES % NT == 0 || p < A_PIECES) {
        const int mb = p / PIECES_PER_BLOCK, within = p % PIECES_PER_BLOCK;
        const long long off = ((long long)mb * n_chunks + c) * T::CH_BYTES + within * 16;
        pa[i] = *reinterpret_cast<const f32x4*>(Ag + off);
        if (DELTA) pd[i] = *reinterpret_cast<const f32x4*>(Dg + off);
      }
    }
  };

  load_tile(u, Umat, row0, 0, N, K, lane);
  if (DELTA) load_tile(w, Wmat, row0, 0, N, K, lane);
  load_A(0);

  for (int c = 0; c < n_chunks; ++c) {
    __syncthreads();  // every wave has finished reading the previous chunk from LDS
#pragma unroll
    for (int i = 0; i < APT; ++i) {
      const int p = tid + i * NT;
      if (A_PIECES % NT == 0 || p < A_PIECES) {
        *reinterpret_cast<f32x4*>(ldsA + p * 16) = pa[i];
        if (DELTA) *reinterpret_cast<f32x4*>(ldsD + p * 16) = pd[i];
      }
    }
    if (do_norm) {
      float q = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) q += (u[j][0] * u[j][0] + u[j][1] * u[j][1]) + (u[j][2] * u[j][2] + u[j][3] * u[j][3]);
      nrm += (double)q;
    }
    stage_tile<BF16>(u, stU, lane);
    if (DELTA) stage_tile<BF16>(w, stW, lane);
    if (c + 1 < n_chunks) {
      load_tile(u, Umat, row0, (c + 1) << 6, N, K, lane);
      if (DELTA) load_tile(w, Wmat, row0, (c + 1) << 6, N, K, lane);
      load_A(c + 1);
    }
    __syncthreads();  // activations of this chunk are visible to all waves

    const int n = lane & 31, h = lane >> 5;
    if (BF16) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bf16x8 bu = *reinterpret_cast<const bf16x8*>(stU + n * T::STAGE_ROW + t * 32 + h * 16);
        bf16x8 bw;
        if (DELTA) bw = *reinterpret_cast<const bf16x8*>(stW + n * T::STAGE_ROW + t * 32 + h * 16);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const bf16x8 ah = *reinterpret_cast<const bf16x8*>(ldsA + ((mb * 4 + t) * 64 + lane) * 16);
          acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bu, acc[mb], 0, 0, 0);
          if (DELTA) {
            const bf16x8 ad = *reinterpret_cast<const bf16x8*>(ldsD + ((mb * 4 + t) * 64 + lane) * 16);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad, bw, acc[mb], 0, 0, 0);
          }
        }
      }
    } else {
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        const f32x4 bu = *reinterpret_cast<const f32x4*>(stU + n * T::STAGE_ROW + (8 * g + 4 * h) * 4);
        f32x4 bw;
        if (DELTA) bw = *reinterpret_cast<const f32x4*>(stW + n * T::STAGE_ROW + (8 * g + 4 * h) * 4);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const f32x4 ah = *reinterpret_cast<const f32x4*>(ldsA + ((mb * 8 + g) * 64 + lane) * 16);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(ah[e], bu[e], acc[mb], 0, 0, 0);
          if (DELTA) {
            const f32x4 ad = *reinterpret_cast<const f32x4*>(ldsD + ((mb * 8 + g) * 64 + lane) * 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(ad[e], bw[e], acc[mb], 0, 0, 0);
          }
        }
      }
    }
  }

  // ---- epilogue.  Accumulator element j of block mb in lane (n, h) is sample row
  // 32 mb + 8 (j/4) + 4 h + j%4 and output feature row0 + n.
  const int n = lane & 31, h = lane >> 5;
  const int feat = row0 + n;
  const bool feat_ok = feat < N;
  float bias = 0.f;
  if (a.b_off >= 0 && feat_ok) bias = P[a.b_off + feat];
  if (do_norm && h == 0) nrm += (double)(bias * bias);

#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int r = 32 * mb + 8 * (j >> 2) + 4 * h + (j & 3);
      const bool ok = feat_ok && r < a.n_r;
      const float val = acc[mb][j] + bias;
      if (is_base) {
        if (ok) a.Z0[(long long)r * N + feat] = val;
        if (!a.last && feat < a.Np) store_tiled<BF16>(a.H_base, r, feat, a.Np, ok ? relu_nan(val) : 0.f);
      } else {
        const float dz = -a.gamma * val;
        if (a.last) {
          if (ok) a.dZ[((long long)s * a.n_r + r) * N + feat] = dz;
        } else if (feat < a.Np) {
          float hv = 0.f, dv = 0.f;
          if (ok) {
            const float z0 = a.Z0[(long long)r * N + feat];
            const float zs = z0 + dz;
            hv = relu_nan(zs);
            // relu(z0 + dz) - relu(z0) without cancellation
            dv = (z0 > 0.f) ? ((dz < -z0) ? -z0 : dz) : hv;
            dv *= a.neg_inv_gamma;
          }
          store_tiled<BF16>(reinterpret_cast<unsigned char*>(a.H_cand) + (long long)s * a.H_stride, r, feat, a.Np, hv);
          store_tiled<BF16>(reinterpret_cast<unsigned char*>(a.Dl_cand) + (long long)s * a.H_stride, r, feat, a.Np, dv);
        }
      }
    }
  }

  if (do_norm) {
    // fixed-order reduction: lanes by xor-shuffle tree, then waves in order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_xor(nrm, off, 64);
    __syncthreads();
    double* red = reinterpret_cast<double*>(lds);
    if (lane == 0) red[wave] = nrm;
    __syncthreads();
    if (tid == 0) {
      double t = 0.0;
      for (int wv = 0; wv < NW; ++wv) t += red[wv];
      a.norm_partials[(long long)s * a.P + a.p_off + nt] = t;
    }
  }
}

template <bool BF16>
__global__ void pack_features_kernel(const float* __restrict__ features, int n_r, int K, int Kp, int n_pad,
                                     void* __restrict__ tiled) {
  const long long total = (long long)n_pad * Kp;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int r = (int)(i / Kp), k = (int)(i % Kp);
    const float v = (r < n_r && k < K) ? features[(long long)r * K + k] : 0.f;
    store_tiled<BF16>(tiled, r, k, Kp, v);
  }
}

template <bool BF16, bool DELTA, int MB, int NW>
hipError_t launch_inst(const LayerArgs& a, hipStream_t stream) {
  using T = Tr<BF16>;
  constexpr int BN = 32 * NW;
  constexpr int lds_bytes = MB * T::CH_BYTES * (DELTA ? 2 : 1) + NW * 32 * T::STAGE_ROW * (DELTA ? 2 : 1);
  static bool attr_set = false;
  if (!attr_set && lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&layer_kernel<BF16, DELTA, MB, NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int n_tiles = (cover_rows(a.N, a.last) + BN - 1) / BN;
  const int grid = ((a.n_src + 7) / 8) * 8 * n_tiles;
  hipLaunchKernelGGL((layer_kernel<BF16, DELTA, MB, NW>), dim3(grid), dim3(64 * NW), lds_bytes, stream, a);
  return hipGetLastError();
}

template <bool BF16, bool DELTA, int MB>
hipError_t launch_nw(const LayerArgs& a, int NW, hipStream_t stream) {
  if (NW == 4) return launch_inst<BF16, DELTA, MB, 4>(a, stream);
  return launch_inst<BF16, DELTA, MB, 1>(a, stream);
}

template <bool BF16, bool DELTA>
hipError_t launch_mb(const LayerArgs& a, int MB, int NW, hipStream_t stream) {
  if (MB == 1) return launch_nw<BF16, DELTA, 1>(a, NW, stream);
  if (MB == 2) return launch_nw<BF16, DELTA, 2>(a, NW, stream);
  return launch_nw<BF16, DELTA, 4>(a, NW, stream);
}

// Waves per workgroup: 4 (128 features per workgroup) when that still gives at
// least two workgroups per compute unit, else 1 (32 features) to spread a narrow
// layer over more compute units.
int pick_nw(int rows, int n_src) {
  const long long wg4 = (long long)((rows + 127) / 128) * n_src;
  return wg4 >= 512 ? 4 : 1;
}

}  // namespace

int layer_tiles(int N, int last, int n_src) {
  const int rows = cover_rows(N, last);
  const int NW = pick_nw(rows, n_src);
  return (rows + 32 * NW - 1) / (32 * NW);
}

hipError_t launch_pack_features(const float* features, int n_r, int K, int Kp, int MB, bool bf16, void* tiled,
                                hipStream_t stream) {
  const int n_pad = 32 * MB;
  const long long total = (long long)n_pad * Kp;
  const int grid = (int)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
  if (bf16) {
    hipLaunchKernelGGL(pack_features_kernel<true>, dim3(grid), dim3(256), 0, stream, features, n_r, K, Kp, n_pad, tiled);
  } else {
    hipLaunchKernelGGL(pack_features_kernel<false>, dim3(grid), dim3(256), 0, stream, features, n_r, K, Kp, n_pad, tiled);
  }
  return hipGetLastError();
}

hipError_t launch_layer(const LayerArgs& a, bool bf16, bool delta, int MB, hipStream_t stream) {
  const int NW = pick_nw(cover_rows(a.N, a.last), a.n_src);
  if (bf16) {
    return delta ? launch_mb<true, true>(a, MB, NW, stream) : launch_mb<true, false>(a, MB, NW, stream);
  }
  return delta ? launch_mb<false, true>(a, MB, NW, stream) : launch_mb<false, false>(a, MB, NW, stream);
}

}  // namespace zeno
