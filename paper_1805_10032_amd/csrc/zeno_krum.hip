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
// krum_gram_kernel<RB> (one or two row blocks, m <= 64; three and four row blocks: krum_gram_shared_kernel
// below): the m <= 32 RB rows are cut into RB row blocks.  A wave owns a
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
  // Two floats at a time: one packed conversion gives both bf16 pieces in one register, and the exact remainder of
  // either float is one instruction, the bf16 dot product of that register with (-1, 0) or (0, -1) added to the
  // float (v_dot2c_f32_bf16: the product with -1 is exact, the product with 0 vanishes, and the sum x - h is
  // representable, so its single rounding changes nothing).  Seven instructions per two floats; taking the pieces'
  // float values out of the packed register with a shift or a mask and subtracting took eleven.
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const float x[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
  // The two constants go through registers: written as immediates, (-1, 0) is emitted as the inline constant -1.0,
  // which this instruction does not read as the bf16 pair (-1, 0) (measured: the remainders then come out wrong).
  unsigned first_bits = 0x0000bf80u, second_bits = 0xbf800000u;
  asm("" : "+s"(first_bits), "+s"(second_bits));
  const bf16x2 minus_first = __builtin_bit_cast(bf16x2, first_bits), minus_second = __builtin_bit_cast(bf16x2, second_bits);
  u32x4 hu, mu, lu;
  auto pack = [](float a, float b) {
    const f32x2 t = {a, b};
    return __builtin_convertvector(t, bf16x2);
  };
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float a = x[2 * i], b = x[2 * i + 1];
    const bf16x2 hp = pack(a, b);
    const float ra = __builtin_amdgcn_fdot2_f32_bf16(hp, minus_first, a, false);
    const float rb = __builtin_amdgcn_fdot2_f32_bf16(hp, minus_second, b, false);
    const bf16x2 mp = pack(ra, rb);
    const float sa = __builtin_amdgcn_fdot2_f32_bf16(mp, minus_first, ra, false);
    const float sb = __builtin_amdgcn_fdot2_f32_bf16(mp, minus_second, rb, false);
    hu[i] = __builtin_bit_cast(unsigned, hp);
    mu[i] = __builtin_bit_cast(unsigned, mp);
    lu[i] = __builtin_bit_cast(unsigned, pack(sa, sb));
  }
  h = __builtin_bit_cast(bf16x8, hu);
  m = __builtin_bit_cast(bf16x8, mu);
  l = __builtin_bit_cast(bf16x8, lu);
}

// CENTER: second pass; runs only if *run_flag != 0 and subtracts row *center from every row.
// NT: streaming loads, where the rows start on 128-byte lines; the 256-byte row segments of other rows share their
// outer lines with the wave's next chunk, which streaming loads would fetch from memory again (dense rows of
// workload 5, m = 64: 3.0 -> 2.8 ms with plain loads; the same switch made the averaging kernel slower, 1.68 -> 1.85 ms,
// and did nothing for the shared-chunk kernel below, so those always stream).
template <int RB, bool CENTER, bool NT>
__global__ __launch_bounds__(64 * kGramWaves, RB == 1 ? 3 : 2) void krum_gram_kernel(const float* __restrict__ G, long long ldg,
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
          v = NT ? load_stream4(p + kq) : *reinterpret_cast<const f32x4_a4*>(p + kq);
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

  static_assert(RB <= 2, "three and four row blocks run krum_gram_shared_kernel");
  {
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

// The Gram kernel for three and four row blocks (64 < m <= 128).  With every wave loading, staging, splitting and
// multiplying its own chunks, and holding all RB (RB + 1) / 2 block products (up to 160 accumulator registers), only
// one wave fits a SIMD and nothing overlaps its vector work and its matrix instructions.  Here the eight waves of a
// workgroup work on ONE chunk at a time, in two roles, one wave of each role per SIMD:
//  * waves 0..3 stage: wave t takes tile t of the chunk (the coalesced loads of krum_gram_kernel, requested four
//    chunks ahead), zeroes the rows beyond m, subtracts the centre row in the second pass, and writes the floats
//    into the chunk's shared buffer, a row per 256 bytes with its 16-byte column groups exclusive-or'ed with the
//    row number (double-buffered: one barrier per chunk);
//  * waves 4..7 multiply, in 16 x 16 blocks (v_mfma_f32_16x16x32_bf16): the m rows are NBL = ceil(m / 16) blocks of
//    16 rows, and only the NBL (NBL + 1) / 2 block pairs a <= b are formed, so rows beyond m cost at most 15 rows of
//    padding and the diagonal blocks waste a 16 x 16 triangle, not a 32 x 32 one (m = 100: 28 pairs x 8 cycles per
//    16 columns and piece product against 10 x 32 with 32-row blocks).  A multiplying wave reads the operand fragment
//    of every block in operand order straight from the staged rows, splits it into the three bf16 pieces and issues
//    the six piece products of its block pairs.  Up to seven blocks (m <= 112) a wave holds all pairs: wave 4 + w
//    takes the 32-column step w & 1 of every second chunk and spreads its products over two barrier intervals, so
//    no block is split twice.  With eight blocks (36 pairs, 144 accumulator registers; it compiles to 252 registers
//    without spills) the same scheme measured no gain (m = 128: 1.69 -> 1.72 ms): there wave 4 + w takes the step
//    w & 1 of every chunk and every second block pair (w >> 1), and both waves of a step split every block.
// The multiplying waves add their accumulators through LDS at the end in a fixed order and write
// the workgroup's partial Gram in the 32 x 32 block layout of krum_gram_kernel (16 x 16 quadrants that are not
// formed, below the diagonal or beyond the last live block, are written as zeros).
// Two things in the staging waves matter as much as the split of roles: the loaded values are first touched when
// their tile is staged (zeroing the rows beyond m right behind the load made every wave wait for the load it had
// just requested), and the steady-state loop has no branch between requesting a tile and staging it four chunks
// later (where paths with different numbers of loads meet, the compiler waits for all of them).
// Measured (MI355X, d = 14.7 M): m = 72 / 96 / 100 / 112 / 128: 0.86 / 1.10 / 1.30 / 1.38 / 1.70-1.75 ms per Krum call
// (m = 72: 5.1 TB/s).  With every block split by both waves of a column step also for m <= 112, same box:
// 0.94 / 1.15 / 1.33 / 1.41 ms (over boxes 0.95 / 1.18 / 1.33-1.40); with the
// eleven-instruction split 1.01 / 1.29 / 1.49 / 1.84 ms.  Before, the staging waves also brought their tile into operand
// order through a private tile and split it, and the multiplying waves read finished pieces: 1.21 / 1.37 / 1.63 /
// 1.88 ms (1.28 / 1.43 / 1.65 / 1.97 ms with 32 x 32 blocks; with krum_gram_kernel<3 or 4> 1.91 / 1.95 / 2.0 / 2.5 ms).
// Timing variants (wrong results, same accesses) without the splitting instructions run at the memory's pace
// (1.16 / 1.17 / 1.37 ms for m = 96 / 100 / 128): the vector instructions of the split add their issue time to the
// matrix instructions' on the same SIMD, whichever wave they sit in.
constexpr int kSharedWaves = 8;

template <int RB>
struct SharedGram {
  static constexpr int PAIRS = RB * (RB + 1) / 2;               // 32 x 32 block pairs of the partial Gram
  static constexpr int TILE_BYTES = 32 * 64 * 4;
  static constexpr int BUF_BYTES = RB * TILE_BYTES;             // one chunk: RB tiles of 32 rows x 64 floats
  static constexpr int LDS_BYTES = 2 * BUF_BYTES;
  static constexpr int MAX_HALF_PAIRS = (2 * RB * (2 * RB + 1) / 2 + 1) / 2;   // 16 x 16 block pairs of one multiplying wave
  static_assert(2 * MAX_HALF_PAIRS * 4 * 64 * 4 <= LDS_BYTES, "the final reduction fits the buffers");
};

template <int RB, int NBL, bool CENTER>
__global__ __launch_bounds__(64 * kSharedWaves) void krum_gram_shared_kernel(const float* __restrict__ G, long long ldg, int m,
                                                                             long long d, float* __restrict__ partial,
                                                                             const int32_t* __restrict__ center,
                                                                             const int32_t* __restrict__ run_flag) {
  using SG = SharedGram<RB>;
  static_assert(NBL == 2 * RB || NBL == 2 * RB - 1, "live 16-row blocks of RB 32-row tiles");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  if (CENTER && *run_flag == 0) return;   // uniform over the launch
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // The 64-column chunks are dealt round-robin to the workgroups: workgroups run at about the same pace, so at any
  // time the chip reads a few contiguous stretches of every row (here c counts the chunks of this workgroup).
  const long long n_chunks = (d + 63) / 64;
  const long long c_end = (n_chunks - blockIdx.x + gridDim.x - 1) / gridDim.x;

  // Both roles pass the same barriers: one after the first chunk is staged, one per chunk in the loop, and those of
  // the final reduction (five where four waves hold partial sums of every block pair, two where two do).
  constexpr bool ALTERNATE = NBL <= 7;
  constexpr int kFinalBarriers = ALTERNATE ? 5 : 2;
  if (wave < 4) {
    // ---- staging waves
    const int t = wave;
    const bool active = t < RB && c_end > 0;
    const float* __restrict__ crow = CENTER ? G + (long long)(*center) * ldg : G;
    const int rsub = lane >> 4, kq = (lane & 15) << 2;
    // FULL: the caller knows that the chunk is complete (no branch on the way to the loads: the compiler counts
    // the loads in flight exactly only along straight-line code, and waits for all of them wherever paths with
    // different numbers of loads meet)
    // (the loaded values are not touched here: rows at or beyond m, which read row m-1, are zeroed and the centre
    // row is subtracted when the tile is staged, so that nothing waits for a load that has just been requested)
    auto load_tile_rows = [&](auto full_c, f32x4 (&u)[8], f32x4& cv, long long c) __attribute__((always_inline)) {
      const long long k0 = (blockIdx.x + c * gridDim.x) * 64;
      const bool k_full = decltype(full_c)::value || k0 + 64 <= d;  // wave-uniform
      if (CENTER) {
        if (k_full) cv = *reinterpret_cast<const f32x4_a4*>(crow + k0 + kq);
        else cv = load4_masked(crow + k0, kq, (int)(d - k0), true);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = 32 * t + 4 * j + rsub;
        const int rc = row < m ? row : m - 1;
        const float* p = G + (long long)rc * ldg + k0;
        if (k_full) u[j] = load_stream4(p + kq);
        else u[j] = load4_masked(p, kq, (int)(d - k0), true);
      }
    };
    auto stage = [&](f32x4 (&u)[8], const f32x4& cv, int buf) __attribute__((always_inline)) {
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 8; ++j) u[j] = (32 * t + 4 * j + rsub < m) ? (CENTER ? u[j] - cv : u[j]) : zero;
      // row r of the tile at r x 256 bytes, its 16-byte column groups exclusive-or'ed with r (the staging tile of
      // the layer kernel): the multiplying waves read it in operand order without bank conflicts
      stage_tile<false>(u, lds + buf * SG::BUF_BYTES + t * SG::TILE_BYTES, lane);
    };
    // four register sets: chunk c sits in set c % 4 and is requested four chunks ahead (four staging waves per compute
    // unit, 8 KB per tile: 128 KB in flight, what it takes to keep the memory system busy at its loaded latency)
    f32x4 u[4][8], cvs[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) cvs[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    using Any = std::false_type;
    using Full = std::true_type;
    if (active) {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (k < c_end) load_tile_rows(Any{}, u[k], cvs[k], k);
      stage(u[0], cvs[0], 0);
      if (4 < c_end) load_tile_rows(Any{}, u[0], cvs[0], 4);
    }
    __syncthreads();
    // four chunks: while the other waves multiply chunk c + k, chunk c + k + 1 is staged and chunk c + k + 5 requested.
    // STEADY: all of those exist and are complete, so nothing in the body branches.
    auto quad = [&](auto steady_c, long long c) __attribute__((always_inline)) {
      constexpr bool STEADY = decltype(steady_c)::value;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (STEADY || c + k < c_end) {
          if (STEADY || (active && c + k + 1 < c_end)) {
            stage(u[(k + 1) & 3], cvs[(k + 1) & 3], (k + 1) & 1);
            if (STEADY) load_tile_rows(Full{}, u[(k + 1) & 3], cvs[(k + 1) & 3], c + k + 5);
            else if (c + k + 5 < c_end) load_tile_rows(Any{}, u[(k + 1) & 3], cvs[(k + 1) & 3], c + k + 5);
          }
          __syncthreads();
        }
      }
    };
    // this workgroup's chunks that are complete (only the last chunk of the matrix can be ragged)
    const long long g_full = d / 64;
    const long long c_full = g_full > blockIdx.x ? (g_full - blockIdx.x + gridDim.x - 1) / gridDim.x : 0;
    long long c = 0;
    if (active) {
      for (; c + 8 < c_full; c += 4) quad(Full{}, c);
    } else {
      // a staging wave without a tile (three row blocks): it only keeps the barriers company
      for (; c + 8 < c_full; c += 4)
        for (int k = 0; k < 4; ++k) __syncthreads();
    }
    for (; c < c_end; c += 4) quad(Any{}, c);
    for (int i = 0; i < kFinalBarriers; ++i) __syncthreads();
    return;
  }

  // ---- multiplying waves
  constexpr int PAIRS16 = NBL * (NBL + 1) / 2;
  if constexpr (ALTERNATE) {
    // Up to seven live row blocks: a wave holds all block pairs (at most 28 x 4 accumulator registers) and all
    // fragments, so no block is split twice.  Wave 4 + w takes the 32-column step w & 1 of every second chunk (w >> 1 its
    // parity) and has two barrier intervals for it: in the chunk's own interval it reads and splits the fragments and
    // issues the first two kinds of piece products, in the next one (from registers, while the other two waves read
    // the next chunk) the remaining four kinds.  The split is the larger half of a multiplying wave's vector work, and
    // vector and matrix instructions of a SIMD do not overlap here; the two intervals then cost about the same.
    const int q = (wave - 4) & 1, parity = (wave - 4) >> 1;
    f32x4 acc[PAIRS16];
#pragma unroll
    for (int i = 0; i < PAIRS16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int frow = lane & 15;
    const int fcol0 = (((8 * q + 2 * (lane >> 4)) ^ frow) & 15) << 4, fcol1 = (((8 * q + 2 * (lane >> 4) + 1) ^ frow) & 15) << 4;
    bf16x8 fh[NBL], fm[NBL], fl[NBL];
    auto fetch = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
      for (int g = 0; g < NBL; ++g) {
        const unsigned char* row = lds + buf * SG::BUF_BYTES + g * (16 * 256) + frow * 256;
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(row + fcol0);
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(row + fcol1);
        split3(v0, v1, fh[g], fm[g], fl[g]);
      }
    };
    // piece products of the kinds [first, last) over all block pairs, kind by kind (the order within a pair's
    // accumulator is that of krum_gram_kernel, smallest first)
    auto products = [&](auto first_c, auto last_c) __attribute__((always_inline)) {
#pragma unroll
      for (int kind = decltype(first_c)::value; kind < decltype(last_c)::value; ++kind) {
        int p = 0;
#pragma unroll
        for (int a = 0; a < NBL; ++a)
#pragma unroll
          for (int b = a; b < NBL; ++b, ++p) {
            const bf16x8 x = kind == 0 ? fl[a] : (kind == 2 || kind == 3) ? fm[a] : fh[a];
            const bf16x8 y = kind == 1 ? fl[b] : (kind == 2 || kind == 4) ? fm[b] : fh[b];
            acc[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, acc[p], 0, 0, 0);
          }
      }
    };
    using K0 = std::integral_constant<int, 0>;
    using K2 = std::integral_constant<int, 2>;
    using K6 = std::integral_constant<int, 6>;
    // Barriers: the one after the first staged chunk; then one per chunk c = 0 .. c_end - 1 at the end of its
    // interval.  A wave of parity 1 sits out interval 0; every wave passes the barrier that ends its chunk's interval
    // and, if that interval is not the last one, the barrier that ends the next.
    __syncthreads();
    if (parity == 1 && c_end > 0) __syncthreads();
    for (long long c = parity; c < c_end; c += 2) {
      fetch((int)(c & 1));
      products(K0{}, K2{});
      __syncthreads();
      products(K2{}, K6{});
      if (c + 1 < c_end) __syncthreads();
    }
    // the four partial sums are added through LDS in the fixed tree (0+2)+(1+3)
    const int w = wave - 4;
    float* red = reinterpret_cast<float*>(lds);
    static_assert(2 * PAIRS16 * 4 * 64 * 4 <= SG::LDS_BYTES, "the final reduction fits the buffers");
    __syncthreads();   // everybody is done with the buffers
    for (int step = 2; step >= 1; step >>= 1) {
      if (w >= step && w < 2 * step) {
#pragma unroll
        for (int p = 0; p < PAIRS16; ++p)
#pragma unroll
          for (int j = 0; j < 4; ++j) red[(((w - step) * PAIRS16 + p) * 4 + j) * 64 + lane] = acc[p][j];
      }
      __syncthreads();
      if (w < step) {
#pragma unroll
        for (int p = 0; p < PAIRS16; ++p)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[p][j] += red[((w * PAIRS16 + p) * 4 + j) * 64 + lane];
      }
      __syncthreads();
    }
    if (w != 0) return;
    // accumulator element j of lane l: row 4 (l / 16) + j of block a, row l % 16 of block b; block pair (a, b) is the
    // quadrant (a % 2, b % 2) of the 32 x 32 block pair (a / 2, b / 2); quadrants nobody forms are written as zeros
    float* out = partial + (long long)blockIdx.x * SG::PAIRS * 1024;
    const int oi = 4 * (lane >> 4), oj = lane & 15;
    auto pair32 = [](int A, int B) { return A * RB - A * (A - 1) / 2 + (B - A); };
#pragma unroll
    for (int A = 0; A < RB; ++A)
#pragma unroll
      for (int B = A; B < RB; ++B)
#pragma unroll
        for (int qa = 0; qa < 2; ++qa)
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            const int a = 2 * A + qa, b = 2 * B + qb;
            const bool formed = a <= b && b < NBL;
            const int p = formed ? a * NBL - a * (a - 1) / 2 + (b - a) : 0;
            float* o = out + pair32(A, B) * 1024 + (qa * 16 + oi) * 32 + qb * 16 + oj;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j * 32] = formed ? acc[p][j] : 0.f;
          }
    return;
  }
  const int q = (wave - 4) & 1;      // 32-column step of every chunk
  const int half = (wave - 4) >> 1;  // block pairs p with p % 2 == half
  f32x4 acc[(PAIRS16 + 1) / 2];
#pragma unroll
  for (int i = 0; i < (PAIRS16 + 1) / 2; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int frow = lane & 15;
  const int fcol0 = (((8 * q + 2 * (lane >> 4)) ^ frow) & 15) << 4, fcol1 = (((8 * q + 2 * (lane >> 4) + 1) ^ frow) & 15) << 4;
  auto multiply = [&](auto half_c, int buf) __attribute__((always_inline)) {
    constexpr int HALF = decltype(half_c)::value;
    // Operand fragment of the 16-row block g and this wave's 32-column step: lane l holds row l % 16, columns
    // 8 (l / 16) .. + 7 of the step, i.e. two 16-byte groups of the staged row, which it splits into the three bf16
    // pieces (the two waves of a column step both split every block: cheaper than passing pieces through LDS).
    bf16x8 fh[NBL], fm[NBL], fl[NBL];
#pragma unroll
    for (int g = 0; g < NBL; ++g) {
      const unsigned char* row = lds + buf * SG::BUF_BYTES + g * (16 * 256) + frow * 256;
      const f32x4 v0 = *reinterpret_cast<const f32x4*>(row + fcol0);
      const f32x4 v1 = *reinterpret_cast<const f32x4*>(row + fcol1);
      split3(v0, v1, fh[g], fm[g], fl[g]);
    }
    // The six piece products of a block pair go to its accumulator in the same order as in krum_gram_kernel
    // (smallest first), but product kind by product kind over all pairs: consecutive matrix instructions then
    // write different accumulators and none waits for the result of the one before it.
#pragma unroll
    for (int kind = 0; kind < 6; ++kind) {
      int p = 0;
#pragma unroll
      for (int a = 0; a < NBL; ++a)
#pragma unroll
        for (int b = a; b < NBL; ++b, ++p) {
          if ((p & 1) != HALF) continue;
          const bf16x8 x = kind == 0 ? fl[a] : (kind == 2 || kind == 3) ? fm[a] : fh[a];
          const bf16x8 y = kind == 1 ? fl[b] : (kind == 2 || kind == 4) ? fm[b] : fh[b];
          acc[p >> 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, acc[p >> 1], 0, 0, 0);
        }
    }
  };
  __syncthreads();
  if (half == 0) {
    for (long long c = 0; c < c_end; ++c) {
      multiply(std::integral_constant<int, 0>{}, (int)(c & 1));
      __syncthreads();
    }
  } else {
    for (long long c = 0; c < c_end; ++c) {
      multiply(std::integral_constant<int, 1>{}, (int)(c & 1));
      __syncthreads();
    }
  }
  // the two column steps of a pair set are added through LDS, step 0 + step 1
  float* red = reinterpret_cast<float*>(lds) + half * (SG::MAX_HALF_PAIRS * 4 * 64);
  __syncthreads();   // everybody is done with the buffers
  if (q == 1) {
#pragma unroll
    for (int i = 0; i < (PAIRS16 + 1) / 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) red[(i * 4 + j) * 64 + lane] = acc[i][j];
  }
  __syncthreads();
  if (q == 1) return;
#pragma unroll
  for (int i = 0; i < (PAIRS16 + 1) / 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] += red[(i * 4 + j) * 64 + lane];
  // accumulator element j of lane l: row 4 (l / 16) + j of block a, row l % 16 of block b; block pair (a, b) is the
  // quadrant (a % 2, b % 2) of the 32 x 32 block pair (a / 2, b / 2)
  float* out = partial + (long long)blockIdx.x * SG::PAIRS * 1024;
  const int oi = 4 * (lane >> 4), oj = lane & 15;
  auto pair32 = [](int A, int B) { return A * RB - A * (A - 1) / 2 + (B - A); };
  {
    int p = 0;
#pragma unroll
    for (int a = 0; a < NBL; ++a)
#pragma unroll
      for (int b = a; b < NBL; ++b, ++p) {
        if ((p & 1) != half) continue;   // (uniform over the wave)
        float* o = out + pair32(a >> 1, b >> 1) * 1024 + ((a & 1) * 16 + oi) * 32 + (b & 1) * 16 + oj;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j * 32] = acc[p >> 1][j];
      }
  }
  if (half == 0) {
    // the quadrants nobody forms: below the diagonal inside a diagonal 32 x 32 block, and those of a block beyond NBL
#pragma unroll
    for (int A = 0; A < RB; ++A)
#pragma unroll
      for (int B = A; B < RB; ++B)
#pragma unroll
        for (int qa = 0; qa < 2; ++qa)
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            const int a = 2 * A + qa, b = 2 * B + qb;
            if (a <= b && b < NBL) continue;
            float* o = out + pair32(A, B) * 1024 + (qa * 16 + oi) * 32 + qb * 16 + oj;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j * 32] = 0.f;
          }
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
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&krum_gram_kernel<RB, false, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(&krum_gram_kernel<RB, false, true>),
                                                     64 * kGramWaves, lds) != hipSuccess || per_cu < 1)
      per_cu = 1;
    return n_cu * per_cu;
  }();
  return cached;
}

int compute_units() {
  static const int n_cu = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
      v = 256;
    return v;
  }();
  return n_cu;
}

// workgroups of the Gram launch: as many as the chip holds at once (three and four row blocks: the eight-wave
// workgroups that share a chunk through LDS, one per compute unit)
int gram_grid(int rb) { return rb == 1 ? gram_resident<1>() : rb == 2 ? gram_resident<2>() : compute_units(); }

inline bool rows_on_lines(const float* G, long long ldg) { return reinterpret_cast<uintptr_t>(G) % 128 == 0 && ldg % 32 == 0; }

template <int RB, int NBL, bool CENTER>
hipError_t launch_gram_shared(const float* G, long long ldg, int m, long long d, float* partial, int grid, const int32_t* center,
                              const int32_t* run_flag, hipStream_t stream) {
  constexpr int lds = SharedGram<RB>::LDS_BYTES;
  static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&krum_gram_shared_kernel<RB, NBL, CENTER>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (attr_err != hipSuccess) return attr_err;
  hipLaunchKernelGGL((krum_gram_shared_kernel<RB, NBL, CENTER>), dim3(grid), dim3(64 * kSharedWaves), lds, stream, G, ldg, m, d,
                     partial, center, run_flag);
  return hipGetLastError();
}

template <int RB, bool CENTER, bool NT>
hipError_t launch_gram_nt(const float* G, long long ldg, int m, long long d, float* partial, int grid, const int32_t* center,
                          const int32_t* run_flag, hipStream_t stream) {
  constexpr int lds = kGramWaves * RB * 32 * 64 * 4;
  static const hipError_t attr_err =
      lds > 48 * 1024 ? hipFuncSetAttribute(reinterpret_cast<const void*>(&krum_gram_kernel<RB, CENTER, NT>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds)
                      : hipSuccess;
  if (attr_err != hipSuccess) return attr_err;
  hipLaunchKernelGGL((krum_gram_kernel<RB, CENTER, NT>), dim3(grid), dim3(64 * kGramWaves), lds, stream, G, ldg, m, d, partial,
                     center, run_flag);
  return hipGetLastError();
}
template <int RB, bool CENTER>
hipError_t launch_gram(const float* G, long long ldg, int m, long long d, float* partial, int grid, const int32_t* center,
                       const int32_t* run_flag, hipStream_t stream) {
  if (rows_on_lines(G, ldg)) return launch_gram_nt<RB, CENTER, true>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  return launch_gram_nt<RB, CENTER, false>(G, ldg, m, d, partial, grid, center, run_flag, stream);
}

template <bool CENTER>
hipError_t launch_gram_rb(int rb, const float* G, long long ldg, int m, long long d, float* partial, int grid,
                          const int32_t* center, const int32_t* run_flag, hipStream_t stream) {
  if (rb == 1) return launch_gram<1, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  if (rb == 2) return launch_gram<2, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  const int nbl = (m + 15) / 16;   // live 16-row blocks
  if (nbl == 5) return launch_gram_shared<3, 5, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  if (nbl == 6) return launch_gram_shared<3, 6, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  if (nbl == 7) return launch_gram_shared<4, 7, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
  return launch_gram_shared<4, 8, CENTER>(G, ldg, m, d, partial, grid, center, run_flag, stream);
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
