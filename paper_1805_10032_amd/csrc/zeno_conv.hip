// Convolutional f_r for the Stochastic Descendant Score (Definition 2; Section 6.1 evaluates
// Zeno on a network of convolutional layers followed by one fully connected layer).
//
// A 3 x 3 convolution with zero padding is a linear layer applied to every output position's
// patch, so the candidates are propagated exactly as through linear layers: for source s
//
//   pass at x:     Z0 = patches(H0) W^T + b,   H0_out = relu(Z0)
//   candidate s:   dZ = -gamma ( patches(H0) U_s^T + patches(D_s) (W - gamma U_s)^T + ub_s ),
//                  D_out = (relu(Z0 + dZ) - relu(Z0)) (-1/gamma)
//
// with W, U_s the kernels [c_out][ky][kx][c_in] of x and of candidate s, H0 the input map of
// the pass at x and D_s the scaled change of candidate s's input map (absent at the first
// convolution).  Nothing is unfolded in memory: a patch element (position, tap, channel) is
// gathered from the NHWC map when a lane needs it as a matrix operand.
//
// One wave owns 32 output positions x 32 output channels in one 32x32 fp32 accumulator block
// (v_mfma_f32_32x32x2_f32, kernel values as the first operand so that a lane is a position and
// its registers are channels), walks the nine taps and, per tap, the input channels eight at a
// time (one 128-bit load per lane and operand feeds four matrix instructions; the tail of a channel
// count that is not a multiple of eight goes two at a time).  Kernels are a few hundred KB per candidate and the maps a few MB, so everything but
// the first touch comes from the caches; the path is bound by instruction issue and latency,
// not by HBM.  The last convolution writes its outputs straight into the matrix-operand
// order of the fully connected layer (rows = samples, columns = (y, x, c)), which the
// streaming layer kernel then consumes.
#include "zeno_layer_impl.h"

namespace zeno {

namespace {

// TW = 3: three waves share one tile and take one kernel row (ky) each; their accumulators are added through
// LDS in the fixed order (0 + 1) + 2 and wave 0 finishes the tile.  Used when the launch has too few tiles
// to occupy the matrix cores otherwise (a wave's 9 c_in / 2 dependent matrix instructions set its pace).
template <bool CAND, int TW>
__global__ __launch_bounds__(64 * TW) void conv_layer_kernel(const ConvArgs a) {
  const ConvLayer& L = a.L;
  const int lane = threadIdx.x & 63, n = lane & 31, h = lane >> 5;
  const int tw = TW > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
  const int ftiles = (L.Cout + 31) / 32;
  const int ft = blockIdx.x % ftiles, rb = blockIdx.x / ftiles;
  const int s = blockIdx.y;
  const int K = 9 * L.Cin;
  const long long rows = (long long)a.n_r * L.Hout * L.Wout;

  const float* __restrict__ P = CAND ? a.G + (long long)s * a.ldg : a.x;
  const bool second = CAND && a.D_in != nullptr;
  const float* __restrict__ Din = second ? a.D_in + (long long)s * a.D_in_stride : nullptr;

  // first operand: kernel row of output channel f, taps and channels contiguous
  const int f = ft * 32 + n;
  const bool f_ok = f < L.Cout;
  const float* __restrict__ Urow = P + L.w_off + (long long)(f_ok ? f : 0) * K;
  const float* __restrict__ Wrow = a.x + L.w_off + (long long)(f_ok ? f : 0) * K;
  // second operand: output position r = (sample, y, x)
  const long long r = (long long)rb * 32 + n;
  const bool r_ok = r < rows;
  const int hw = L.Hout * L.Wout;
  const int smp = (int)((r_ok ? r : 0) / hw), pos = (int)((r_ok ? r : 0) % hw);
  const int oy = pos / L.Wout, ox = pos % L.Wout;

  f32x16 acc;
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.f;
  const float neg_gamma = -a.gamma;

  for (int tap = (TW > 1 ? 3 * tw : 0); tap < (TW > 1 ? 3 * tw + 3 : 9); ++tap) {
    const int ky = tap / 3, kx = tap % 3;
    const int iy = oy * L.stride + ky - 1, ix = ox * L.stride + kx - 1;
    const bool p_ok = r_ok && iy >= 0 && iy < L.Hin && ix >= 0 && ix < L.Win;
    const long long moff = (((long long)smp * L.Hin + (p_ok ? iy : 0)) * L.Win + (p_ok ? ix : 0)) * L.Cin;
    const float* __restrict__ hp = a.H0_in + moff;
    const float* __restrict__ dp = second ? Din + moff : nullptr;
    const float* __restrict__ up = Urow + tap * L.Cin;
    const float* __restrict__ wp = Wrow + tap * L.Cin;
    // channels two at a time: this lane's half h takes channel c0 + h
    int c0 = 0;
    // Eight channels at a time: each lane loads FOUR consecutive channels of its kernel row / its position with
    // one 128-bit load (half h takes channels c0 + 4h .. c0 + 4h + 3) and feeds four matrix instructions, the
    // i-th of which contracts the channel pair (c0 + i, c0 + 4 + i).  Two such groups are loaded ahead of
    // their instructions.  A wave walks its operands alone, so the loads in flight set its pace.
    auto group8 = [&](auto ng_c) __attribute__((always_inline)) {
      constexpr int NG = decltype(ng_c)::value;
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      f32x4 u[NG], b1[NG], w[NG], b2[NG];
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int c = c0 + 8 * g + 4 * h;
        u[g] = f_ok ? *reinterpret_cast<const f32x4_a4*>(up + c) : zero;
        b1[g] = p_ok ? *reinterpret_cast<const f32x4_a4*>(hp + c) : zero;
        if (second) {
          w[g] = f_ok ? *reinterpret_cast<const f32x4_a4*>(wp + c) : zero;
          b2[g] = p_ok ? *reinterpret_cast<const f32x4_a4*>(dp + c) : zero;
        }
      }
#pragma unroll
      for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(u[g][i], b1[g][i], acc, 0, 0, 0);
          if (second)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_fmaf(neg_gamma, u[g][i], w[g][i]), b2[g][i], acc, 0, 0, 0);
        }
    };
    for (; c0 + 16 <= L.Cin; c0 += 16) group8(std::integral_constant<int, 2>{});
    for (; c0 + 8 <= L.Cin; c0 += 8) group8(std::integral_constant<int, 1>{});
    for (; c0 < L.Cin; c0 += 2) {
      const int c = c0 + h;
      const bool c_ok = c < L.Cin;
      const float u = (f_ok && c_ok) ? up[c] : 0.f;
      const float b1 = (p_ok && c_ok) ? hp[c] : 0.f;
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(u, b1, acc, 0, 0, 0);
      if (second) {
        const float w = (f_ok && c_ok) ? wp[c] : 0.f;
        const float b2 = (p_ok && c_ok) ? dp[c] : 0.f;
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_fmaf(neg_gamma, u, w), b2, acc, 0, 0, 0);
      }
    }
  }

  if (TW > 1) {
    __shared__ float red[2][16][64];
    if (tw > 0) {
#pragma unroll
      for (int j = 0; j < 16; ++j) red[tw - 1][j][lane] = acc[j];
    }
    __syncthreads();
    if (tw > 0) return;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = (acc[j] + red[0][j][lane]) + red[1][j][lane];
  }
  // accumulator element j of lane (n, h): position r (this lane's), output channel ft*32 + 8 (j/4) + 4 h + j%4
  if (!r_ok) return;
  float* __restrict__ out = CAND ? a.out + (long long)s * a.out_stride : a.out;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int fo = ft * 32 + 8 * (j >> 2) + 4 * h + (j & 3);
    if (fo >= L.Cout) continue;
    const float bias = L.b_off >= 0 ? P[L.b_off + fo] : 0.f;
    const float val = acc[j] + bias;
    float res;
    if (!CAND) {
      a.Z0[r * L.Cout + fo] = val;
      res = relu_nan(val);
    } else {
      const float dz = -a.gamma * val;
      const float z0 = a.Z0[r * L.Cout + fo];
      const float hr = relu_nan(z0 + dz);
      // relu(z0 + dz) - relu(z0) without cancellation
      const float dd = (z0 > 0.f) ? ((dz < -z0) ? -z0 : dz) : hr;
      res = dd * a.neg_inv_gamma;
    }
    if (a.tiled_out) {
      out[tiled_index<false>(smp, pos * L.Cout + fo, a.Kp_fc)] = res;
    } else {
      out[r * L.Cout + fo] = res;
    }
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ p, long long n16) {
  const uint4 z = {0u, 0u, 0u, 0u};
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (long long)gridDim.x * blockDim.x) p[i] = z;
}

// Sum of squares of a slice of every candidate, piece `blk` of n_blocks, fixed order: a thread sums
// its strided elements in fp64, lanes by xor-shuffle tree, waves in order.
__global__ __launch_bounds__(256) void sumsq_kernel(const float* __restrict__ G, long long ldg, long long begin,
                                                    long long count, double* __restrict__ partials, int P, int p_off) {
  __shared__ double red[4];
  const int s = blockIdx.y, blk = blockIdx.x, nb = gridDim.x;
  const long long lo = count * blk / nb, hi = count * (blk + 1) / nb;
  const float* __restrict__ row = G + (long long)s * ldg + begin;
  double t = 0.0;
  for (long long i = lo + threadIdx.x; i < hi; i += 256) {
    const double v = (double)row[i];
    t += v * v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
  __syncthreads();
  if (threadIdx.x == 0) partials[(long long)s * P + p_off + blk] = ((red[0] + red[1]) + red[2]) + red[3];
}

}  // namespace

hipError_t launch_conv(const ConvArgs& a, hipStream_t stream) {
  const long long rows = (long long)a.n_r * a.L.Hout * a.L.Wout;
  const long long row_blocks = (rows + 31) / 32;
  const int ftiles = (a.L.Cout + 31) / 32;
  const int sources = a.n_cand > 0 ? a.n_cand : 1;
  const dim3 grid((unsigned)(row_blocks * ftiles), sources);
  // one wave per tile when there are tiles enough for every SIMD of the chip twice over, else three
  const bool wide = row_blocks * ftiles * sources >= 2048;
  if (a.n_cand > 0) {
    if (wide) hipLaunchKernelGGL((conv_layer_kernel<true, 1>), grid, dim3(64), 0, stream, a);
    else hipLaunchKernelGGL((conv_layer_kernel<true, 3>), grid, dim3(192), 0, stream, a);
  } else {
    if (wide) hipLaunchKernelGGL((conv_layer_kernel<false, 1>), grid, dim3(64), 0, stream, a);
    else hipLaunchKernelGGL((conv_layer_kernel<false, 3>), grid, dim3(192), 0, stream, a);
  }
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream) {
  const long long n16 = (long long)(bytes / 16);   // the slots are multiples of 256 bytes
  if (n16 == 0) return hipSuccess;
  const long long want = (n16 + 255) / 256;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)(want > 4096 ? 4096 : want)), dim3(256), 0, stream,
                     reinterpret_cast<uint4*>(p), n16);
  return hipGetLastError();
}

hipError_t launch_sumsq(const float* G, long long ldg, int m, long long begin, long long count, int n_blocks,
                        double* partials, int P, int p_off, hipStream_t stream) {
  hipLaunchKernelGGL(sumsq_kernel, dim3(n_blocks, m), dim3(256), 0, stream, G, ldg, begin, count, partials, P, p_off);
  return hipGetLastError();
}

}  // namespace zeno
