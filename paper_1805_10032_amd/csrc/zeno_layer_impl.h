// Streaming layer kernel of the Stochastic Descendant Score (Definition 2).
//
// For one linear layer l and every source s of the launch (candidate rows G[s],
// s < m, and the current parameters x as source m) a workgroup owns BN = 32*NW
// output features and streams the corresponding rows of that source's weight
// block from HBM exactly once, K-chunk by K-chunk:
//
//   source m (pass at x):   Z0   = H0 W^T + b                           (pre-activations at x)
//   source s < m:           dZ_s = -gamma ( H0 U_s^T + D_s (W - gamma U_s)^T + ub_s )
//
// where H0 are the input activations of the pass at x (shared by all candidates), U_s / ub_s
// candidate s's weight / bias block, and D_s = (H_s - H0) * (-1/gamma) the scaled change of the
// candidate's input activations (absent at the first layer, where H_s = H0 = the batch).  Only
// D_s is stored per candidate.  With H_s = H0 - gamma D_s the candidate's own product
// H_s U_s^T + D_s W^T equals H0 U_s^T + D_s (W - gamma U_s)^T: the first product runs on the
// shared activations, and the second on the perturbed weights, which a wave forms in registers
// for the 32 x 64 tile it has just staged and never stores.  dZ_s is the change of the
// pre-activations caused by moving x to x - gamma u_s, so f_r(x) - f_r(x - gamma u) is later
// obtained without subtracting two nearly equal losses.  ||u_s||^2 is accumulated from the same
// registers that feed the matrix cores.
//
// Matrix-core mapping (wave64): each wave owns 32 output features (the rows of its
// 32x32 accumulator blocks, i.e. the weight tile is the FIRST operand) and all
// MB*32 sample rows (the columns = lanes), so that the results leave the
// accumulators already in the order the next layer's operand is stored in.
//  * U tile (32 features x 64 k, fp32 in HBM): fully coalesced 128-bit loads (4
//    rows x 256 B per instruction, scalar base + per-lane offset), two chunks in
//    flight per wave; converted and passed through a wave-private, XOR-swizzled
//    LDS tile to reach the operand layout (lane = feature, 8 consecutive k).
//  * Activation operands H_s, D_s: stored in global memory already in operand
//    order ("tiled"), copied asynchronously global -> LDS (no registers) into a
//    double buffer and shared by the waves of the workgroup: one barrier per chunk.
//  * W operand of the second product: written in operand order by the pass at x,
//    loaded straight into registers, where gamma times the staged U operand (same
//    layout) is subtracted from it.
#ifndef ZENO_LAYER_IMPL_H_
#define ZENO_LAYER_IMPL_H_

#include <type_traits>

#include "zeno_internal.h"

namespace zeno {

namespace {

typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int kSrcChunk = 16;  // sources per scheduling unit (one feature tile each)

template <bool BF16>
struct Tr;
template <>
struct Tr<true> {
  static constexpr int ESIZE = 2;
  static constexpr int CH_BYTES = 32 * 64 * 2;  // one 32-row block of a 64-wide K chunk, tiled operand
};
template <>
struct Tr<false> {
  static constexpr int ESIZE = 4;
  static constexpr int CH_BYTES = 32 * 64 * 4;
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

// Four consecutive columns k0..k0+3 (k0 a multiple of 4) of row r of a tiled
// operand: they are adjacent in memory (8 bytes as bf16, 16 bytes as fp32).
template <bool BF16>
__device__ inline void store_tiled4(void* base, int r, int k0, int Kp, const f32x4& v) {
  const long long idx = tiled_index<BF16>(r, k0, Kp);
  // write-through stores (system-scope bit): the results are not kept as dirty lines
  // in the L2, where the streaming weight loads would have to displace them.  The
  // s_nop after the 128-bit store is required: the hardware still reads the data
  // registers of a store wider than 64 bits for two more cycles, and the compiler,
  // which adds these wait states to its own stores, does not look inside assembly.
  if (BF16) {
    bf16x4 t;
    t[0] = (__bf16)v[0]; t[1] = (__bf16)v[1]; t[2] = (__bf16)v[2]; t[3] = (__bf16)v[3];
    asm volatile("global_store_dwordx2 %0, %1, off sc1" ::"v"(reinterpret_cast<__bf16*>(base) + idx), "v"(t) : "memory");
  } else {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(reinterpret_cast<float*>(base) + idx), "v"(v) : "memory");
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

// Store v[0..3] to row[k..k+3], dropping the elements at or beyond K (4-byte aligned row).
__device__ inline void store4_masked(float* __restrict__ row, int k, int K, const f32x4& v) {
  if (k + 4 <= K) {
    f4u t;
    t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
    *reinterpret_cast<f4u*>(row + k) = t;
  } else {
    if (k < K) row[k] = v[0];
    if (k + 1 < K) row[k + 1] = v[1];
    if (k + 2 < K) row[k + 2] = v[2];
  }
}

// Load the wave's 32 x 64 weight tile: instruction j covers rows 4j..4j+3, 256
// contiguous bytes each.  `tile` is the wave-uniform address of element (row0, k0);
// `lane_off` = (lane/16)*K + 4*(lane%16) is the lane's element offset inside it.
// MODE 1: the whole tile lies inside the matrix (no masking code is generated).
// MODE 2: every K chunk is complete but some rows lie at or beyond N: they read row
// N-1 instead (always in bounds) and the caller discards them, so that a ragged last
// feature tile runs the same straight-line loop as a full one.
// MODE 0: K is not a multiple of the chunk width (element-wise guards in the last chunk).
// NT: streaming loads that do not keep the lines in the caches.  Only chosen when
// every 256-byte row segment starts on a 128-byte line: a line that two load
// instructions share would otherwise be fetched from memory twice.
template <int MODE, bool NT>
__device__ inline void load_tile(f32x4 (&u)[8], const float* __restrict__ tile, unsigned lane_off, int row0, int k0,
                                 int N, int K, int lane) {
  if (MODE != 0) {
    if (MODE == 1) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (NT) {
          u[j] = load_stream4(tile + (long long)(4 * j) * K + lane_off);
        } else {
          u[j] = *reinterpret_cast<const f32x4_a4*>(tile + (long long)(4 * j) * K + lane_off);
        }
      }
    } else {
      const int rsub = lane >> 4, kq = (lane & 15) << 2;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = row0 + 4 * j + rsub;
        const int rel = (row < N ? row : N - 1) - row0;   // may be negative: the tile starts beyond the matrix
        const float* p = tile + (long long)rel * K + kq;
        if (NT) {
          u[j] = load_stream4(p);
        } else {
          u[j] = *reinterpret_cast<const f32x4_a4*>(p);
        }
      }
    }
  } else {
    // Ragged tile.  Rows beyond the matrix read row N-1 instead (always in bounds)
    // and are zeroed afterwards; only the last K chunk of a width that is not a
    // multiple of 64 takes the element-wise path.
    const int rsub = lane >> 4, kq = (lane & 15) << 2;
    const bool k_full = k0 + 64 <= K;  // wave-uniform
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row = row0 + 4 * j + rsub;
      const int back = row < N ? 0 : row - (N - 1);
      const float* p = tile + (long long)(4 * j + rsub - back) * K;
      f32x4 v;
      if (k_full) {
        v = *reinterpret_cast<const f32x4_a4*>(p + kq);
      } else {
        v = load4_masked(p, kq, K - k0, true);
      }
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      u[j] = row < N ? v : zero;
    }
  }
}

// Wave-private staging tile, unpadded and XOR-swizzled on 16-byte segments so that
// both the row-wise writes and the operand reads (lane = row) are conflict-free.
template <bool BF16>
__device__ inline void stage_tile(const f32x4 (&u)[8], unsigned char* st, int lane) {
  const int rsub = lane >> 4, kq = lane & 15;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int r = 4 * j + rsub;
    if (BF16) {
      const bf16x4 h = __builtin_convertvector(u[j], bf16x4);
      *reinterpret_cast<bf16x4*>(st + r * 128 + ((((kq >> 1) ^ (r >> 1)) & 7) << 4) + ((kq & 1) << 3)) = h;
    } else {
      *reinterpret_cast<f32x4*>(st + r * 256 + (((kq ^ r) & 15) << 4)) = u[j];
    }
  }
}

// Tiles of the shifted column grid (see RING below) whose first or last columns fall outside the row: the
// lanes there read the row's first or last four elements instead (in bounds, and in a line that the tile's
// valid columns need anyway) and deliver zeros.  kfirst is the column of the tile's first element, K a
// multiple of 4 like kfirst, so a lane's four columns are all inside or all outside.
template <int MODE, bool NT>
__device__ inline void load_tile_edge(f32x4 (&u)[8], const float* __restrict__ Urow0, int kfirst, int row0, int N, int K,
                                      int lane) {
  const int rsub = lane >> 4, k = kfirst + ((lane & 15) << 2);
  const bool ok = k >= 0 && k < K;
  const int kk = k < 0 ? 0 : (k < K ? k : K - 4);
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = row0 + 4 * j + rsub;
    const int rel = ((MODE == 2 && row >= N) ? N - 1 : row) - row0;
    const float* p = Urow0 + (long long)rel * K + kk;
    f32x4 v;
    if (NT) {
      v = load_stream4(p);
    } else {
      v = *reinterpret_cast<const f32x4_a4*>(p);
    }
    u[j] = ok ? v : zero;
  }
}

// The same for rows that are only 8-byte aligned (the shift sigma and K are even): a lane's four columns may be
// half inside the row, so each half is loaded (64 bits) and masked on its own; a half that lies outside reads
// the row's first or last two elements instead.
template <int MODE, bool NT>
__device__ inline void load_tile_edge2(f32x4 (&u)[8], const float* __restrict__ Urow0, int kfirst, int row0, int N, int K,
                                       int lane) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef f32x2 f32x2_a4 __attribute__((aligned(4)));
  const int rsub = lane >> 4, k = kfirst + ((lane & 15) << 2);
  const bool ok0 = k >= 0 && k < K, ok1 = k + 2 >= 0 && k + 2 < K;
  const int k0 = k < 0 ? 0 : (k < K ? k : K - 2);
  const int k1 = k + 2 < 0 ? 0 : (k + 2 < K ? k + 2 : K - 2);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = row0 + 4 * j + rsub;
    const int rel = ((MODE == 2 && row >= N) ? N - 1 : row) - row0;
    const float* p = Urow0 + (long long)rel * K;
    f32x2 a, b;
    if (NT) {
      a = __builtin_nontemporal_load(reinterpret_cast<const f32x2_a4*>(p + k0));
      b = __builtin_nontemporal_load(reinterpret_cast<const f32x2_a4*>(p + k1));
    } else {
      a = *reinterpret_cast<const f32x2_a4*>(p + k0);
      b = *reinterpret_cast<const f32x2_a4*>(p + k1);
    }
    u[j][0] = ok0 ? a[0] : 0.f;
    u[j][1] = ok0 ? a[1] : 0.f;
    u[j][2] = ok1 ? b[0] : 0.f;
    u[j][3] = ok1 ? b[1] : 0.f;
  }
}

// Staging ring of the shifted column grid (bf16): two staging tiles of the ordinary layout, the first for
// the columns whose bit 6 is clear, the second for the others.  A tile of the shifted grid starts sigma
// columns before a multiple of 64, so its first sigma columns go to one half and the rest to the other.
// ring_w: the lane's byte offset for row lane / 16 of an EVEN tile; an odd tile flips the half, and the offset for
// row 4 i + lane / 16 is ring_w exclusive-or a constant: the row bits (i * 512) and the swizzle bits
// ((2 i mod 8) * 16) of i touch no bit that the lane's part sets differently.  One register instead of eight, in a
// kernel that has none to spare.
__device__ inline unsigned ring_offset(int lane, int sigma) {
  const int rsub = lane >> 4, kq = lane & 15;
  const int col = (4 * kq - sigma) & 63;            // column inside its block of 64
  const int kp = col >> 2;
  const unsigned half = 4 * kq < sigma ? 4096u : 0u;   // columns before the tile's own block of 64
  return half + rsub * 128 + ((((kp >> 1) ^ (rsub >> 1)) & 7) << 4) + ((kp & 1) << 3);
}
template <bool ODD>
__device__ inline void stage_ring(const f32x4 (&u)[8], unsigned char* st, unsigned ring_w) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const bf16x4 h = __builtin_convertvector(u[i], bf16x4);
    // the constant is hidden from the optimiser, which would otherwise hoist the eight offsets out of the
    // K loop and keep them in eight registers again
    unsigned ci = ((unsigned)(i * 512) | (unsigned)(((2 * i) & 7) << 4)) ^ (ODD ? 4096u : 0u);
    asm volatile("" : "+s"(ci));
    *reinterpret_cast<bf16x4*>(st + (ring_w ^ ci)) = h;
  }
}

// Rows that are only 8-byte aligned: sigma is even, so the two column pairs of a lane's four may fall into
// different 8-byte pieces, 16-byte segments or halves of the ring; each pair is written on its own (32 bits).
// The byte offset of a pair for row 4 i + lane / 16 is its offset for row lane / 16 exclusive-or a constant:
// the row bits (i * 512) and the swizzle bits ((2 i mod 8) * 16) of i touch no bit that the lane's part sets
// differently, so two registers hold the offsets of all eight rows.
__device__ inline void ring_offsets2(unsigned (&ring_p)[2], int lane, int sigma) {
  const int rsub = lane >> 4, kq = lane & 15;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int t = 4 * kq + 2 * p;                       // first column of the pair inside the tile
    const int col = (t - sigma) & 63;                   // column inside its block of 64
    const unsigned half = t < sigma ? 4096u : 0u;       // columns before the tile's own block of 64
    ring_p[p] = half + rsub * 128 + ((((col >> 3) ^ (rsub >> 1)) & 7) << 4) + ((col & 7) << 1);
  }
  // A 32-bit write is served 32 lanes at a time, i.e. two rows of the staging tile, and two adjacent rows (128 bytes
  // apart, same swizzle) fall on the same banks when they write the same pair (same position inside the 16-byte
  // segments).  The lanes of the odd rows therefore write their pairs in the other order (stage_ring2 swaps the
  // data the same way): the two rows of a half-instruction then use different 4-byte positions of every segment.
  if (rsub & 1) {
    const unsigned t = ring_p[0];
    ring_p[0] = ring_p[1];
    ring_p[1] = t;
  }
}
template <bool ODD>
__device__ inline void stage_ring2(const f32x4 (&u)[8], unsigned char* st, const unsigned (&ring_p)[2], bool swap) {
  unsigned flip = ODD ? 4096u : 0u;
  asm volatile("" : "+s"(flip));
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const bf16x4 h = __builtin_convertvector(u[i], bf16x4);
    const unsigned ci = (unsigned)(i * 512) | (unsigned)(((2 * i) & 7) << 4);
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 w = __builtin_bit_cast(u32x2, h);   // w[0]: columns 0, 1 of the lane's four; w[1]: columns 2, 3
    // swap (the lanes of the odd rows): ring_p[0] is the offset of the second pair, ring_p[1] of the first
    *reinterpret_cast<unsigned*>(st + (ring_p[0] ^ ci ^ flip)) = swap ? w[1] : w[0];
    *reinterpret_cast<unsigned*>(st + (ring_p[1] ^ ci ^ flip)) = swap ? w[0] : w[1];
  }
}

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt in
// bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
template <int N>
__device__ inline void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Asynchronous 16-byte-per-lane copy from global memory straight into LDS: lane i's
// 16 bytes at `src` (a per-lane address) land at dst + 16 i, dst wave-uniform.  The
// instruction is issued through inline assembly on purpose.  The compiler's own
// wait-count bookkeeping treats such a copy as a possible writer of every LDS
// address and then drains ALL outstanding loads (vmcnt(0)) before the next LDS
// read, which would also drain the weight tiles that are meant to stay in flight
// across chunks.  Issued this way the copy is invisible to that bookkeeping; the
// kernel waits for it explicitly (wait_vmcnt, loads complete in order) before the
// workgroup barrier that publishes the buffer.  Hidden loads only make the
// compiler's own counts for its ordinary loads stricter than needed, never laxer.
// m0 (the LDS base of the copy) cannot be declared clobbered: the compiler treats it as a
// reserved register and ignores such a declaration (with a warning).  The statement
// therefore saves m0 in a scalar register of its own and restores it behind the copy, so
// whatever the compiler keeps in m0 survives.
__device__ inline void lds_dma16(const unsigned char* src, unsigned char* dst) {
  const unsigned lds_off = (unsigned)(uintptr_t)(lptr_t)dst;  // byte offset inside the workgroup's LDS
  unsigned saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(src), "s"(lds_off)
               : "memory");
}

// LDS layout of a workgroup: [activation chunk buffers (one or two)] [one staging
// tile per wave].  (Nothing else: with 4 row blocks, bf16 operands, the second product and
// four waves the layout is exactly 80 KB, and two such workgroups share a compute unit.)
template <bool BF16, bool DELTA, int MB, int NW, int RING = 0>
struct Lds {
  using T = Tr<BF16>;
  static constexpr int A_BYTES = MB * T::CH_BYTES;            // one operand, one chunk
  static constexpr int AD_BYTES = A_BYTES * (DELTA ? 2 : 1);  // H (and D), one chunk
  static constexpr int STAGE_BYTES = 32 * 64 * T::ESIZE * (RING ? 2 : 1);   // RING: two tiles' worth of columns
  static constexpr bool DBUF = 2 * AD_BYTES + NW * STAGE_BYTES <= 128 * 1024;
  static constexpr int STAGE_OFF = AD_BYTES * (DBUF ? 2 : 1);
  static constexpr int TOTAL = STAGE_OFF + NW * STAGE_BYTES;
};

// KS > 1 (launches of one-wave tiles, NW == 1): the KS waves of a workgroup own the SAME
// 32 features and split the K range between them, each with a private copy of the LDS
// layout and no barrier inside the loop; the partial accumulators (and the partial
// squared norms) are summed through LDS in a fixed order at the end and wave 0 writes
// the results.  A launch of the pass at x has only N/32 feature tiles, and a narrow
// layer (ten classes) only one tile per candidate: far too few single waves to keep
// enough loads in flight, and each of them would walk all of K alone, one chunk's
// latency after the other.  This multiplies the waves by KS and divides the walk.
//
// RING (bf16 operands, NW > 1): the shifted column grid for rows that do not start on 128-byte lines (a dense
// G[m x d]).  With K a multiple of 64 and 16-byte aligned rows every row of a wave's tile starts the same
// sigma columns (a multiple of 4) past a line.  A 64-column tile that starts at column 64 j would then cover
// three lines per row and share the outer two with its neighbours: they would come from memory twice.  Here
// tile j starts at column 64 j - sigma instead, on a line, so that every line is requested once (and can be
// streamed); the tiles are staged into a ring of 128 columns at (column mod 128), one tile ahead of the
// products, which read their 64 columns at the unshifted positions.  Nothing else knows of the shift.  The
// first tile's columns before the row and the last (extra) tile's columns behind it are masked.
//
// TAIL (eight-wave workgroups): the launch ends with the tiles of its last a.tail_cand candidates (may be none) and
// of the pass at x, if it rides along, cut into a.tail_slices K slices each.  A launch whose workgroups do not fill their last
// round of resident slots would run that round at a fraction of the chip; cut into slices the same tiles are
// several times as many workgroups, each a fraction as long.  The slices of a tile hand their partial accumulators
// over through memory as the K slices of one-wave tiles do (last workgroup to arrive adds them in slice order).
template <bool BF16, bool DELTA, int MB, int NW, bool NT, int KS, int RING = 0, bool TAIL = false>
__global__ __launch_bounds__(64 * NW * KS) void layer_kernel(const LayerArgs a) {
  static_assert(KS == 1 || NW == 1, "K is only split in one-tile workgroups");
  using T = Tr<BF16>;
  using LD = Lds<BF16, DELTA, MB, NW, RING>;
  static_assert(!TAIL || (NW == 8 && KS == 1 && LD::DBUF), "sliced tails exist for double-buffered eight-wave workgroups");
  static_assert(!RING || (BF16 && KS == 1 && NW > 1 && LD::DBUF), "the shifted grid exists for wide bf16 workgroups with double buffers");
  static_assert(KS == 1 || LD::DBUF, "the single-buffer loop has workgroup barriers, which waves with different K ranges cannot share");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];
  constexpr int BN = 32 * NW;
  constexpr int A_BYTES = LD::A_BYTES;
  constexpr int AD_BYTES = LD::AD_BYTES;
  constexpr int AD_KB = AD_BYTES / 1024;               // 1 KB async copies per chunk
  constexpr int A_KB = A_BYTES / 1024;
  constexpr int BLOCK_KB = T::CH_BYTES / 1024;
  constexpr int STAGE_BYTES = LD::STAGE_BYTES;
  constexpr bool DBUF = LD::DBUF;
  constexpr int COPIES = (AD_KB + NW - 1) / NW;        // async copies issued per wave per chunk
  constexpr int WREGS = BF16 ? 4 : 8;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave = KS > 1 ? 0 : wave_id;   // feature sub-tile of this wave inside the workgroup's tile
  const int kw = KS > 1 ? wave_id : 0;     // which part of K this wave sums
  unsigned char* lds = lds_all + kw * LD::TOTAL;
  unsigned char* stU = lds + LD::STAGE_OFF + wave * STAGE_BYTES;

  // Which job: the leading base_blocks block indices run the pass at x (one
  // feature tile each), the rest the candidates.
  // Candidates: workgroups are dealt round-robin to the 8 XCDs (blockIdx % 8), each
  // with its own L2.  The work is cut into units of one feature tile x a chunk of up
  // to kSrcChunk candidates; units go round-robin to the XCDs and the workgroups of
  // a unit occupy consecutive slots of their XCD.  The workgroups that run together
  // on an XCD therefore stream the SAME rows of W (second product) at about the
  // same time and share them through that L2, while everything that is private to
  // a candidate (its activations) is reused inside the workgroup through LDS.
  // TAIL: the block indices from a.main_blocks on are the sliced tiles, numbered [tiles of the pass at x]
  // [tail candidates x tiles], a.tail_slices consecutive blocks per tile; the pass at x has no leading blocks then.
  bool is_base = (int)blockIdx.x < a.base_blocks;
  int tail_tile = -1;   // >= 0: this workgroup runs one K slice of that tile of the tail
  int tail_base_tiles = 0;
  if constexpr (TAIL) {
    if ((int)blockIdx.x >= a.main_blocks) {
      tail_tile = ((int)blockIdx.x - a.main_blocks) / a.tail_slices;
      tail_base_tiles = a.has_base ? (cover_rows(a.bj.N, a.bj.last) + BN - 1) / BN : 0;
      is_base = tail_tile < tail_base_tiles;
    }
  }
  const LayerJob& J = is_base ? a.bj : a.cj;
  const int N = J.N, K = J.K, last = J.last, Np = J.Np;
  const int n_chunks = J.Kp >> 6;
  const int n_tiles = (cover_rows(N, last) + BN - 1) / BN;
  int nt, s = 0;
  // K slice of this workgroup: a launch of one-wave tiles whose tiles do not fill the chip well splits K
  // over k_slices workgroups per tile (on top of, or instead of, the split over the KS waves of a workgroup)
  int ks = 0;
  const int n_slices = (TAIL && tail_tile >= 0) ? a.tail_slices : (NW == 1 && a.k_slices > 1) ? a.k_slices : 1;
  const int n_main = TAIL ? a.n_cand - a.tail_cand : a.n_cand;   // candidates whose tiles run whole
  if (TAIL && tail_tile >= 0) {
    ks = ((int)blockIdx.x - a.main_blocks) % n_slices;
    if (is_base) {
      nt = tail_tile;
    } else {
      const int g = tail_tile - tail_base_tiles;
      nt = g % n_tiles;
      s = n_main + g / n_tiles;
      if (s >= a.n_cand) return;
    }
  } else if (is_base) {
    nt = blockIdx.x / n_slices;
    ks = blockIdx.x % n_slices;
    if (nt >= n_tiles) return;
  } else {
    int bid = blockIdx.x - a.base_blocks;
    ks = bid % n_slices;
    bid /= n_slices;
    const int cc = n_main < kSrcChunk ? n_main : kSrcChunk;
    const int n_cchunks = (n_main + cc - 1) / cc;
    const int xcd = bid & 7, slot = bid >> 3;
    const int unit = (slot / cc) * 8 + xcd;
    if (unit >= n_tiles * n_cchunks) return;
    nt = unit / n_cchunks;
    s = (unit % n_cchunks) * cc + slot % cc;
    if (s >= n_main) return;
  }
  const float* __restrict__ P = is_base ? a.x : a.G + (long long)s * a.ldg;
  const int row0 = nt * BN + wave * 32;
  const float* __restrict__ Urow0 = P + J.w_off + (long long)row0 * K;  // wave-uniform
  const unsigned lane_off = (unsigned)(lane >> 4) * (unsigned)K + ((lane & 15) << 2);
  const bool full_rows = row0 + 32 <= N;
  // RING: columns between the line a row starts in and the row's first element (the same for all rows of the tile)
  const int sigma = RING ? __builtin_amdgcn_readfirstlane((int)((reinterpret_cast<uintptr_t>(Urow0) & 127) >> 2)) : 0;
  const float* __restrict__ Uring = Urow0 - sigma;   // tile j of the shifted grid starts at Uring + 64 j
  unsigned ring_w = 0, ring_p[2];
  if constexpr (RING == 1) ring_w = ring_offset(lane, sigma);
  if constexpr (RING == 2) ring_offsets2(ring_p, lane, sigma);

  const unsigned char* Ag = reinterpret_cast<const unsigned char*>(J.A_base);
  // The pass at x has no second product: its D operand is a harmless alias of H
  // and its products are skipped.
  const bool has_delta = DELTA && !is_base;
  const unsigned char* Dg = has_delta ? reinterpret_cast<const unsigned char*>(a.D_cand) + (long long)s * a.A_stride : Ag;

  const bool pack = is_base && J.Wt != nullptr;
  unsigned char* Wt_wave = reinterpret_cast<unsigned char*>(J.Wt) +
                           ((long long)(row0 >> 5) * n_chunks * WREGS * 64 + lane) * 16;
  // The main loop exists in six versions chosen per wave: full tile / full K with some
  // rows beyond the matrix (both: straight-line loads, and the in-order completion of
  // loads lets a chunk wait for exactly its own activation copies) / ragged in K, and BASE (pass at x: no second product, writes W in operand order) or
  // candidate.
  const bool all_full = (K & 63) == 0;
  // this workgroup's chunks (slices of wide workgroups start at even chunks)
  const int cs0 = (n_chunks * ks / n_slices) & (NW > 1 ? ~1 : ~0);
  const int cs1 = ks + 1 == n_slices ? n_chunks : (n_chunks * (ks + 1) / n_slices) & (NW > 1 ? ~1 : ~0);
  const int c_begin = NW == 1 ? cs0 + (cs1 - cs0) * kw / KS : TAIL ? cs0 : 0;
  const int c_end = NW == 1 ? cs0 + (cs1 - cs0) * (kw + 1) / KS : TAIL ? cs1 : n_chunks;

  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[mb][j] = 0.f;

  const bool do_norm = (a.norm_partials != nullptr) && !is_base;
  double nrm = 0.0;

  f32x4 u0[8], u1[8];
  f32x4 w0[WREGS], w1[WREGS];
  float bias_lane = 0.f;

  // Asynchronous copy of chunk c of the tiled activation operands into LDS buffer
  // `buf`: AD_KB pieces of 1 KB (64 lanes x 16 B land at consecutive LDS addresses),
  // dealt round-robin to the waves.
  auto copy_AD = [&](int c, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < COPIES; ++i) {
      const int q = wave + i * NW;
      if (AD_KB % NW == 0 || q < AD_KB) {
        const int op = q / A_KB, piece = q % A_KB;
        const int mb = piece / BLOCK_KB, within = piece % BLOCK_KB;
        const unsigned char* src = (op ? Dg : Ag) + ((long long)mb * n_chunks + c) * T::CH_BYTES + within * 1024 + lane * 16;
        unsigned char* dst = lds + buf * AD_BYTES + q * 1024;
        lds_dma16(src, dst);
      }
    }
  };
  const float neg_gamma = -a.gamma;
  // Operand of the second product: W - gamma U for one k-step, from the W operand (operand-order
  // copy written by the pass at x) and the staged U operand, which share one register layout.
  // One fused multiply-add per element in fp32, then the operand rounding.
  auto perturbed_w = [&](const f32x4& wv, const f32x4& uv) __attribute__((always_inline)) {
    f32x4 out;
    if (BF16) {
      const bf16x8 wb = __builtin_bit_cast(bf16x8, wv), ub = __builtin_bit_cast(bf16x8, uv);
      bf16x8 r;
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = (__bf16)__builtin_fmaf(neg_gamma, (float)ub[e], (float)wb[e]);
      out = __builtin_bit_cast(f32x4, r);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) out[e] = __builtin_fmaf(neg_gamma, uv[e], wv[e]);
    }
    return out;
  };
  auto load_W = [&](f32x4 (&w)[WREGS], int c) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < WREGS; ++r)
      w[r] = *reinterpret_cast<const f32x4*>(Wt_wave + ((long long)c * WREGS + r) * 1024);
  };

  // A weight tile that has arrived in registers: rows beyond the matrix are discarded, its share of
  // ||u||^2 is taken, and it is converted and staged (RING: as an even or odd tile of the shifted grid).
  // count: the tile's share of ||u||^2 belongs to this workgroup (a K slice on the shifted grid also stages the
  // first tile of the next slice, which that slice counts).
  auto take_tile = [&](auto full_c, auto odd_c, f32x4 (&u)[8], bool count) __attribute__((always_inline)) {
    constexpr int MODE = decltype(full_c)::value;
    if (MODE == 2) {
      // rows beyond the matrix were read from row N-1: discard them
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 8; ++i) u[i] = (row0 + 4 * i + (lane >> 4) < N) ? u[i] : zero;
    }
    if (do_norm && count) {
      float q = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) q += (u[i][0] * u[i][0] + u[i][1] * u[i][1]) + (u[i][2] * u[i][2] + u[i][3] * u[i][3]);
      nrm += (double)q;
    }
    if constexpr (RING == 1) {
      stage_ring<decltype(odd_c)::value>(u, stU, ring_w);
    } else if constexpr (RING == 2) {
      stage_ring2<decltype(odd_c)::value>(u, stU, ring_p, (lane & 16) != 0);
    } else {
      stage_tile<BF16>(u, stU, lane);
    }
  };
  // Tile j of the shifted grid (RING), j >= 1: the last one (j == n_chunks) lies partly behind the row.
  auto load_ring = [&](auto full_c, f32x4 (&u)[8], int j) __attribute__((always_inline)) {
    constexpr int MODE = decltype(full_c)::value;
    if (j < n_chunks) {
      load_tile<MODE, NT>(u, Uring + (j << 6), lane_off, row0, j << 6, N, K, lane);
    } else if (sigma > 0) {
      if constexpr (RING == 2) load_tile_edge2<MODE, NT>(u, Urow0, 64 * j - sigma, row0, N, K, lane);
      else load_tile_edge<MODE, NT>(u, Urow0, 64 * j - sigma, row0, N, K, lane);
    } else {
      // rows that start on a line: the grid is not shifted and there is no tile behind the last chunk
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 8; ++i) u[i] = zero;
    }
  };

  // One K chunk.  Its weight tile sits in registers u (loaded two chunks ago); its
  // activation operands were copied into LDS buffer c&1 during the previous chunk.
  // Issue order per chunk: copies(c+1), U(c+2), [matrix products of c], W(c+2).
  // STEADY: the caller guarantees c + 2 < n_chunks, so every load of the chunk is
  // unconditional.  That matters for more than the saved branches: the compiler
  // derives its wait counts from the worst path through the loop, and a path on
  // which the later tile was NOT requested makes it wait for all loads at the top
  // of every chunk, i.e. no tile would stay in flight across a chunk.
  // odd_c: the parity of c in wide workgroups (selects the activation buffer, and with RING the half of the staging ring, at compile time).
  auto chunk = [&](auto full_c, auto base_c, auto steady_c, auto odd_c, f32x4 (&u)[8], f32x4 (&w)[WREGS], int c)
                   __attribute__((always_inline)) {
    constexpr bool ODD = decltype(odd_c)::value;
    constexpr int MODE = decltype(full_c)::value;
    constexpr bool FULL = MODE != 0;
    constexpr bool BASE = decltype(base_c)::value;   // this workgroup runs the pass at x
    constexpr bool STEADY = decltype(steady_c)::value;
    constexpr bool SECOND = DELTA && !BASE;           // second product D W^T present
    // wide workgroups start at an even chunk, so the parity of c, and with it every LDS address of the chunk,
    // is a compile-time constant; waves that split K may start anywhere
    const int buf = DBUF ? (NW > 1 ? (ODD ? 1 : 0) : (c & 1)) : 0;
    // RING: u holds tile c + 1 of the shifted grid, staged one chunk ahead of the products
    take_tile(full_c, std::integral_constant<bool, !ODD>{}, u, !(RING && TAIL) || c + 1 < c_end || c_end == n_chunks);
    if (DBUF) {
      // copies(c) were issued before U(c+1) [8 loads] and W(c+1) [WREGS loads]; the
      // last chunk has no such loads behind its copies and waits for everything
      // (the stores of the pass at x, which writes W in operand order, share the counter;
      // they can only make this wait longer, never let it pass early)
      // (shifted grid: the tile requested behind copies(c) is tile c + 2, which is not requested at all where it
      // would lie wholly behind rows that start on a line; then the copies are the newest but WREGS loads)
      if (FULL && (STEADY || (c + 1 < c_end && (!RING || c + 2 < n_chunks || sigma > 0)))) {
        wait_vmcnt<8 + (SECOND ? WREGS : 0)>();
      } else {
        wait_vmcnt<0>();
      }
      if (KS == 1) {
        __syncthreads();  // copies of every wave have landed; everyone is done with buffer buf^1
      } else {
        asm volatile("" ::: "memory");  // private buffers: only the compiler must not move LDS reads above the wait
      }
      // Issue priorities of a wave inside a chunk: highest while it requests the next copies and weight
      // tiles (memory requests leave as early as possible), raised during the matrix products, lowest
      // while it converts and stages a tile.  Of the two waves that share a SIMD the one that is behind
      // (still in its products while the other already stages the next tile) is served first, and it is
      // the one every other wave of the workgroup will wait for at the next barrier.
      __builtin_amdgcn_s_setprio(3);
      if (STEADY || c + 1 < c_end) copy_AD(c + 1, buf ^ 1);
      __builtin_amdgcn_sched_barrier(0);  // the wait above counts on the copies being issued before the next loads
    } else {
      __syncthreads();  // single buffer: everyone is done with the previous chunk
      copy_AD(c, 0);
      wait_vmcnt<0>();
      __syncthreads();
    }
    if constexpr (RING) {
      if (STEADY) load_tile<MODE, NT>(u, Uring + ((c + 3) << 6), lane_off, row0, (c + 3) << 6, N, K, lane);
      else if (c + 3 <= c_end) load_ring(full_c, u, c + 3);
    } else {
      if (STEADY || c + 2 < c_end) load_tile<MODE, NT>(u, Urow0 + ((c + 2) << 6), lane_off, row0, (c + 2) << 6, N, K, lane);
    }

    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
    // Matrix products of this chunk in groups of MB products that share one B
    // operand (k-step t, operand H or D).  The scheduler is fenced so that the LDS
    // reads of group g+1 are issued right behind the products of group g.
    const unsigned char* bufA = lds + buf * AD_BYTES;
    const unsigned char* bufD = bufA + A_BYTES;
    const int n = lane & 31, h = lane >> 5;
    constexpr int OPS = DELTA ? 2 : 1;
    constexpr int KSTEPS = BF16 ? 4 : 8;   // operand k-steps per chunk (16 k / 8 k each)
    constexpr int NG = KSTEPS * OPS;
    auto read_group = [&](f32x4 (&fr)[MB], int g) __attribute__((always_inline)) {
      const int t = g / OPS, op = g % OPS;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        fr[mb] = *reinterpret_cast<const f32x4*>((op ? bufD : bufA) + ((mb * KSTEPS + t) * 64 + lane) * 16);
    };
    auto read_b = [&](int t) __attribute__((always_inline)) {
      if (RING) return *reinterpret_cast<const f32x4*>(stU + (ODD ? 4096 : 0) + n * 128 + ((((2 * t + h) ^ (n >> 1)) & 7) << 4));
      if (BF16) return *reinterpret_cast<const f32x4*>(stU + n * 128 + ((((2 * t + h) ^ (n >> 1)) & 7) << 4));
      return *reinterpret_cast<const f32x4*>(stU + n * 256 + ((((2 * t + h) ^ n) & 15) << 4));
    };
    f32x4 fr[NG][MB];
    f32x4 bq[KSTEPS];
    bq[0] = read_b(0);
    read_group(fr[0], 0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int t = g / OPS, op = g % OPS;
      __builtin_amdgcn_sched_barrier(0);
      const f32x4 bv = op ? (SECOND ? perturbed_w(w[t], bq[t]) : w[t]) : bq[t];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        if (op == 1 && !SECOND) break;  // the pass at x has no second product
        if (BF16) {
          acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bv),
                                                            __builtin_bit_cast(bf16x8, fr[g][mb]), acc[mb], 0, 0, 0);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[e], fr[g][mb][e], acc[mb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // the reads of the next group are issued behind this group's products and
      // complete while the matrix pipeline works through them
      if (g + 1 < NG) {
        read_group(fr[g + 1], g + 1);
        if ((g + 1) % OPS == 0) bq[(g + 1) / OPS] = read_b((g + 1) / OPS);
      }
      if (BASE && pack && op == 0) *reinterpret_cast<f32x4*>(Wt_wave + ((long long)c * WREGS + t) * 1024) = bq[t];
    }
    __builtin_amdgcn_s_setprio(0);
    if (SECOND && (STEADY || c + 2 < c_end)) load_W(w, c + 2);
  };

  auto run = [&](auto full_c, auto base_c) __attribute__((always_inline)) {
    constexpr int MODE = decltype(full_c)::value;
    constexpr bool FULL = MODE != 0;
    constexpr bool SECOND = DELTA && !decltype(base_c)::value;
    // The wave's 32 bias values are requested first of all (lane i < 32 keeps feature row0 + i's),
    // so that the epilogue does not start with a round trip to memory.
    if (J.b_off >= 0 && lane < 32 && row0 + lane < N) bias_lane = P[J.b_off + row0 + lane];
    __builtin_amdgcn_sched_barrier(0);
    if (DBUF) copy_AD(c_begin, NW > 1 ? 0 : c_begin & 1);
    __builtin_amdgcn_sched_barrier(0);
    int c = c_begin;
    const float* Ufirst = Urow0 + (c_begin << 6);
    if constexpr (RING) {
      // the first two tiles of the shifted grid (c is even: wide workgroups and their K slices start at even chunks);
      // the first is staged here, every chunk then stages the tile after its own.  The products of chunk j read
      // tiles j and j + 1, so a K slice that ends before the row does still needs tile c_end.
      if (c > 0) load_tile<MODE, NT>(u0, Uring + (c << 6), lane_off, row0, c << 6, N, K, lane);
      else if constexpr (RING == 2) load_tile_edge2<MODE, NT>(u0, Urow0, -sigma, row0, N, K, lane);
      else load_tile_edge<MODE, NT>(u0, Urow0, -sigma, row0, N, K, lane);
      load_ring(full_c, u1, c + 1);
      if (SECOND) {
        load_W(w0, c);
        if (c + 1 < c_end) load_W(w1, c + 1);
      }
      take_tile(full_c, std::false_type{}, u0, true);
      if (c + 2 <= c_end) load_ring(full_c, u0, c + 2);
      // steady state: chunks whose tile three ahead lies fully inside the rows (c is even here)
      for (; c + 4 < c_end; c += 2) {
        chunk(full_c, base_c, std::true_type{}, std::false_type{}, u1, w0, c);
        chunk(full_c, base_c, std::true_type{}, std::true_type{}, u0, w1, c + 1);
      }
      for (; c < c_end; c += 2) {
        chunk(full_c, base_c, std::false_type{}, std::false_type{}, u1, w0, c);
        if (c + 1 < c_end) chunk(full_c, base_c, std::false_type{}, std::true_type{}, u0, w1, c + 1);
      }
    } else {
    if (FULL && DBUF && c_end - c_begin >= 4) {
      // steady state: pairs of chunks whose loads (two chunks ahead) all exist
      load_tile<MODE, NT>(u0, Ufirst, lane_off, row0, c_begin << 6, N, K, lane);
      load_tile<MODE, NT>(u1, Ufirst + 64, lane_off, row0, (c_begin + 1) << 6, N, K, lane);
      if (SECOND) {
        load_W(w0, c_begin);
        load_W(w1, c_begin + 1);
      }
      for (; c + 3 < c_end; c += 2) {
        chunk(full_c, base_c, std::true_type{}, std::false_type{}, u0, w0, c);
        chunk(full_c, base_c, std::true_type{}, std::true_type{}, u1, w1, c + 1);
      }
    } else {
      if (c_begin < c_end) load_tile<MODE, NT>(u0, Ufirst, lane_off, row0, c_begin << 6, N, K, lane);
      if (c_begin + 1 < c_end) load_tile<MODE, NT>(u1, Ufirst + 64, lane_off, row0, (c_begin + 1) << 6, N, K, lane);
      if (SECOND) {
        load_W(w0, c_begin);
        if (c_begin + 1 < c_end) load_W(w1, c_begin + 1);
      }
    }
    // the last two or three chunks (all of them for a short K): every load is conditional
    for (; c < c_end; c += 2) {
      chunk(full_c, base_c, std::false_type{}, std::false_type{}, u0, w0, c);
      if (c + 1 < c_end) chunk(full_c, base_c, std::false_type{}, std::true_type{}, u1, w1, c + 1);
    }
    if (KS > 1) wait_vmcnt<0>();  // a wave with an empty K range still has its first copy in flight
    }
  };
  using M0 = std::integral_constant<int, 0>;
  using M1 = std::integral_constant<int, 1>;
  using M2 = std::integral_constant<int, 2>;
  if (is_base) {
    if (all_full && full_rows) run(M1{}, std::true_type{});
    else if (all_full || RING) run(M2{}, std::true_type{});   // the shifted grid is only launched for K a multiple of 64
    else run(M0{}, std::true_type{});
  } else {
    if (all_full && full_rows) run(M1{}, std::false_type{});
    else if (all_full || RING) run(M2{}, std::false_type{});
    else run(M0{}, std::false_type{});
  }

  if (KS > 1) {
    // sum the KS partial accumulators in a fixed tree: (0+2)+(1+3) for KS = 4
    float* red = reinterpret_cast<float*>(lds_all);
    for (int step = KS / 2; step >= 1; step >>= 1) {
      __syncthreads();  // all waves are out of their loops / done reading the previous round
      if (kw >= step && kw < 2 * step) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int j = 0; j < 16; ++j) red[(((kw - step) * MB + mb) * 16 + j) * 64 + lane] = acc[mb][j];
      }
      __syncthreads();
      if (kw < step) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int j = 0; j < 16; ++j) acc[mb][j] += red[((kw * MB + mb) * 16 + j) * 64 + lane];
      }
    }
    if (do_norm) {
      // the waves' partial squared norms: each wave sums its lanes, wave 0 adds the totals
      // in wave order and carries the result in lane 0 into the reduction after the epilogue
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) nrm += __shfl_xor(nrm, off, 64);
      double* nred = reinterpret_cast<double*>(lds_all + LD::TOTAL);  // wave 1's layout, idle by now and beyond `red`
      if (kw != 0 && lane == 0) nred[kw] = nrm;
      __syncthreads();
      if (kw == 0) {
        double t = nrm;
        for (int w = 1; w < KS; ++w) t += nred[w];
        nrm = lane == 0 ? t : 0.0;
      }
    }
    if (kw != 0) return;
  }
  bool finish = true;   // this workgroup completes the tile: epilogue and results
  if ((NW == 1 || TAIL) && n_slices > 1) {
    if (NW == 1 && KS == 1 && do_norm) {
      // one wave per workgroup: bring its share of ||u||^2 to lane 0, as the K split over waves does
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) nrm += __shfl_xor(nrm, off, 64);
      nrm = lane == 0 ? nrm : 0.0;
    }
    // K was also split over workgroups: publish this workgroup's partial accumulators, and let the last
    // workgroup of the tile to arrive add all of them, in slice order whoever it is, and finish the tile
    // layout: per slice and wave MB*4 pieces of 64 lanes x 16 bytes (accumulator registers 4q..4q+3 of block mb)
    constexpr int WAVE_FLOATS = MB * 16 * 64;
    const long long slice_stride = (long long)NW * WAVE_FLOATS;
    // the tile this workgroup shares (TAIL: the sliced tiles are numbered as their blocks are)
    const long long grp = TAIL ? tail_tile : is_base ? nt : a.slice_group0 + (long long)s * n_tiles + nt;
    float* part = a.slice_partials + grp * n_slices * slice_stride + wave * WAVE_FLOATS;   // this wave's features
    float* mine = part + ks * slice_stride;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 v = {acc[mb][4 * q], acc[mb][4 * q + 1], acc[mb][4 * q + 2], acc[mb][4 * q + 3]};
        // written through to memory (system scope): the compute units' L2 caches are per XCD and the
        // workgroup that adds the partials may sit on another one
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(mine + ((mb * 4 + q) * 64 + lane) * 4), "v"(v) : "memory");
      }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the partials have reached memory before the arrival is counted
    unsigned arrived = 0;
    if constexpr (NW == 1) {
      if (lane == 0) arrived = __hip_atomic_fetch_add(&a.slice_counters[grp], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      // one arrival per workgroup, counted when the partials of all its waves are out; the count reaches the
      // other waves through LDS (the activation buffers are idle: every wave has left the loop by the barrier)
      __syncthreads();
      unsigned* flag = reinterpret_cast<unsigned*>(lds_all);
      if (tid == 0) *flag = __hip_atomic_fetch_add(&a.slice_counters[grp], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __syncthreads();
      arrived = *flag;
    }
    arrived = __builtin_amdgcn_readfirstlane(arrived);
    if (arrived != (unsigned)(n_slices - 1)) {
      if constexpr (NW == 1) {
        // not the last one: only this slice's share of ||u||^2 is left to deliver (lane 0 holds it)
        if (do_norm && lane == 0) a.norm_partials[(long long)s * a.P + a.p_off + nt * n_slices + ks] = nrm;
        return;
      }
      finish = false;   // wide workgroups: the waves still add up their share of ||u||^2 below
    } else {
    // The other workgroups' partials are read with system-scope loads (they bypass the caches on the way,
    // as the stores did, so no cache has to be written back or invalidated).  A round trip to memory is
    // long while other workgroups stream at full rate, so the loads of several slices (up to 64 registers'
    // worth) are issued together and completed by one wait; the wait statements name the loaded registers
    // as operands so that no use of them can be scheduled ahead of it.  The sum is taken in slice order
    // whoever adds it; this workgroup's own slice comes from its registers (bit-identical to what it stored).
    // slices per round trip: 4, 2 or 1; sliced tails with one or two row blocks have the registers for 8 or 4
    constexpr int BATCH = (TAIL && MB < 4 ? 8 : 4) / MB;
    f32x16 total[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int j = 0; j < 16; ++j) total[mb][j] = 0.f;
    for (int q0 = 0; q0 < n_slices; q0 += BATCH) {
      f32x4 t[BATCH][MB][4];
#pragma unroll
      for (int i = 0; i < BATCH; ++i) {
        const int q = q0 + i;
        if (q < n_slices && q != ks) {   // uniform over the wave
          const float* other = part + q * slice_stride;
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1" : "=v"(t[i][mb][r]) : "v"(other + ((mb * 4 + r) * 64 + lane) * 4) : "memory");
        } else {
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 4; ++r) t[i][mb][r] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int i = 0; i < BATCH; ++i)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          asm volatile("" : "+v"(t[i][mb][0]), "+v"(t[i][mb][1]), "+v"(t[i][mb][2]), "+v"(t[i][mb][3])::"memory");
#pragma unroll
      for (int i = 0; i < BATCH; ++i) {
        const int q = q0 + i;
        if (q >= n_slices) break;
        if (q == ks) {
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) total[mb][j] += acc[mb][j];
        } else {
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
              for (int e = 0; e < 4; ++e) total[mb][4 * r + e] += t[i][mb][r][e];
        }
      }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = total[mb];
    if (NW == 1 ? lane == 0 : tid == 0)
      __hip_atomic_store(&a.slice_counters[grp], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next pass
    }
  }

  // ---- epilogue.  The weight tile is the first operand of the products, so the
  // accumulators hold features along the registers and samples along the lanes:
  // element j of block mb in lane (n, h) is sample row 32 mb + n and output feature
  // row0 + 8 (j/4) + 4 h + j%4.  Four consecutive features of one sample are
  // adjacent in the tiled operand of the next layer, so a lane stores them as one
  // piece and a wave's store instruction covers one contiguous 512 B / 1 KB run.
  if (finish) {
  const int n = lane & 31, h = lane >> 5;
  f32x4 bias[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
#pragma unroll
    for (int i = 0; i < 4; ++i) bias[q][i] = __shfl(bias_lane, 8 * q + 4 * h + i, 64);   // loaded before the main loop
    // every feature of the tile sits in exactly one of the two lanes with n == 0
    if (do_norm && n == 0)
      nrm += (double)((bias[q][0] * bias[q][0] + bias[q][1] * bias[q][1]) + (bias[q][2] * bias[q][2] + bias[q][3] * bias[q][3]));
  }

  if (full_rows) {
    // All 32 features of the wave exist: no per-element guards.  Rows beyond the
    // batch read row n_r-1 instead (in bounds) and are masked afterwards, so every
    // load is unconditional and all of them are in flight together.
    const bool hidden_cand = !is_base && !last;
    f32x4 z0v[MB][4];
    if (hidden_cand) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int r = 32 * mb + n;
        const int rc = r < a.n_r ? r : a.n_r - 1;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          z0v[mb][q] = *reinterpret_cast<const f32x4_a4*>(J.Z0 + (long long)rc * N + row0 + 8 * q + 4 * h);
      }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int r = 32 * mb + n;
      const bool row_ok = r < a.n_r;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int f0 = row0 + 8 * q + 4 * h;
        f32x4 val;
#pragma unroll
        for (int i = 0; i < 4; ++i) val[i] = acc[mb][4 * q + i] + bias[q][i];
        if (is_base) {
          if (row_ok) *reinterpret_cast<f32x4_a4*>(J.Z0 + (long long)r * N + f0) = val;
          if (!last) {
            f32x4 hv;
#pragma unroll
            for (int i = 0; i < 4; ++i) hv[i] = row_ok ? relu_nan(val[i]) : 0.f;
            store_tiled4<BF16>(J.H_base, r, f0, Np, hv);
          }
        } else {
          f32x4 dz;
#pragma unroll
          for (int i = 0; i < 4; ++i) dz[i] = -a.gamma * val[i];
          if (last) {
            if (row_ok) *reinterpret_cast<f32x4_a4*>(a.dZ + ((long long)s * a.n_r + r) * N + f0) = dz;
          } else {
            f32x4 dv;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float z0 = z0v[mb][q][i];
              const float hr = relu_nan(z0 + dz[i]);
              // relu(z0 + dz) - relu(z0) without cancellation
              const float dd = (z0 > 0.f) ? ((dz[i] < -z0) ? -z0 : dz[i]) : hr;
              dv[i] = row_ok ? dd * a.neg_inv_gamma : 0.f;
            }
            store_tiled4<BF16>(reinterpret_cast<unsigned char*>(a.Dl_cand) + (long long)s * a.H_stride, r, f0, Np, dv);
          }
        }
      }
    }
  } else {
    // ragged tile: per-element guards
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int r = 32 * mb + n;
      const bool row_ok = r < a.n_r;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int f0 = row0 + 8 * q + 4 * h;
        f32x4 val;
#pragma unroll
        for (int i = 0; i < 4; ++i) val[i] = acc[mb][4 * q + i] + bias[q][i];
        if (is_base) {
          if (row_ok) store4_masked(J.Z0 + (long long)r * N, f0, N, val);
          if (!last && f0 < Np) {
            f32x4 hv;
#pragma unroll
            for (int i = 0; i < 4; ++i) hv[i] = (row_ok && f0 + i < N) ? relu_nan(val[i]) : 0.f;
            store_tiled4<BF16>(J.H_base, r, f0, Np, hv);
          }
        } else {
          f32x4 dz;
#pragma unroll
          for (int i = 0; i < 4; ++i) dz[i] = -a.gamma * val[i];
          if (last) {
            if (row_ok) store4_masked(a.dZ + ((long long)s * a.n_r + r) * N, f0, N, dz);
          } else if (f0 < Np) {
            const f32x4 z0 = load4_masked(J.Z0 + (long long)r * N, f0, N, row_ok);
            f32x4 dv;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const bool ok = row_ok && f0 + i < N;
              const float hr = relu_nan(z0[i] + dz[i]);
              // relu(z0 + dz) - relu(z0) without cancellation
              const float dd = (z0[i] > 0.f) ? ((dz[i] < -z0[i]) ? -z0[i] : dz[i]) : hr;
              dv[i] = ok ? dd * a.neg_inv_gamma : 0.f;
            }
            store_tiled4<BF16>(reinterpret_cast<unsigned char*>(a.Dl_cand) + (long long)s * a.H_stride, r, f0, Np, dv);
          }
        }
      }
    }
  }

  }   // finish

  if (do_norm) {
    // fixed-order reduction: lanes by xor-shuffle tree, then waves in order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_xor(nrm, off, 64);
    if (NW == 1) {
      // only one wave is left, and it holds the sum over this workgroup's chunks
      if (lane == 0) a.norm_partials[(long long)s * a.P + a.p_off + nt * n_slices + ks] = nrm;
    } else {
      __syncthreads();
      double* red = reinterpret_cast<double*>(lds);
      if (lane == 0) red[wave] = nrm;
      __syncthreads();
      if (tid == 0) {
        double t = 0.0;
        for (int wv = 0; wv < NW; ++wv) t += red[wv];
        // the sliced tiles of a launch's tail have a range of slots of their own, one per (tile, slice)
        const int slot = (TAIL && tail_tile >= 0) ? a.tail_p_off + nt * n_slices + ks : a.p_off + nt;
        a.norm_partials[(long long)s * a.P + slot] = t;
      }
    }
  }
}

template <bool BF16>
__global__ void pack_features_kernel(const float* __restrict__ features, int n_r, int K, int Kp, int n_pad,
                                     void* __restrict__ tiled, unsigned int* __restrict__ counters, int n_counters,
                                     double* __restrict__ zero, long long n_zero) {
  const long long total = (long long)n_pad * Kp;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n_counters; i += (long long)gridDim.x * blockDim.x)
    counters[i] = 0u;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n_zero; i += (long long)gridDim.x * blockDim.x)
    zero[i] = 0.0;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int r = (int)(i / Kp), k = (int)(i % Kp);
    const float v = (r < n_r && k < K) ? features[(long long)r * K + k] : 0.f;
    store_tiled<BF16>(tiled, r, k, Kp, v);
  }
}

int job_tiles(const LayerJob& j, int BN) { return (cover_rows(j.N, j.last) + BN - 1) / BN; }

template <bool BF16, bool DELTA, int MB, int NW, bool NT, int KS = 1, int RING = 0, bool TAIL = false>
hipError_t launch_inst(LayerArgs a, hipStream_t stream, LaunchShape* shape) {
  constexpr int BN = 32 * NW;
  if (shape != nullptr) {
    shape->waves = NW;
    shape->k_split = KS;
    shape->k_slices = TAIL ? a.tail_slices : NW == 1 && a.k_slices > 1 ? a.k_slices : 1;
    shape->streaming = RING ? 1 + RING : NT ? 1 : 0;
    shape->row_blocks = MB;
  }
  constexpr int lds_bytes = Lds<BF16, DELTA, MB, NW, RING>::TOTAL * KS;
  // once per process and instantiation (initialisation of a local static is thread-safe)
  static const hipError_t attr_err =
      lds_bytes > 48 * 1024 ? hipFuncSetAttribute(reinterpret_cast<const void*>(&layer_kernel<BF16, DELTA, MB, NW, NT, KS, RING, TAIL>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes)
                            : hipSuccess;
  if (attr_err != hipSuccess) return attr_err;
  // K slices (one-wave tiles only) come with the caller's plan; they need the partial and counter buffers
  if (NW != 1 || a.k_slices < 1) a.k_slices = 1;
  if (a.k_slices > 1 && (a.slice_partials == nullptr || a.slice_counters == nullptr)) return hipErrorInvalidValue;
  if (!TAIL) a.tail_cand = a.tail_slices = 0;
  if (TAIL && (a.tail_cand < 0 || a.tail_cand >= a.n_cand || (a.tail_cand == 0 && !a.has_base) || a.tail_slices < 2 ||
               a.slice_partials == nullptr || a.slice_counters == nullptr))
    return hipErrorInvalidValue;
  // TAIL: the pass at x has no leading blocks, its tiles are sliced like the tail candidates'
  a.base_blocks = (a.has_base && !TAIL) ? (job_tiles(a.bj, BN) * a.k_slices + 7) / 8 * 8 : 0;
  const int n_main = a.n_cand - a.tail_cand;
  int cand_blocks = 0;
  if (n_main > 0) {
    const int cc = n_main < kSrcChunk ? n_main : kSrcChunk;
    const int units = job_tiles(a.cj, BN) * ((n_main + cc - 1) / cc);
    cand_blocks = ((units + 7) / 8) * 8 * cc * a.k_slices;
  }
  a.main_blocks = a.base_blocks + cand_blocks;
  int tail_blocks = 0;
  if (TAIL) {
    const long long tiles = (a.has_base ? job_tiles(a.bj, BN) : 0) + (long long)job_tiles(a.cj, BN) * a.tail_cand;
    // every slice keeps at least two chunks of every job; the hand-over buffers hold all sliced tiles
    if ((a.cj.Kp >> 6) < 2 * a.tail_slices || (a.has_base && (a.bj.Kp >> 6) < 2 * a.tail_slices) ||
        tiles * a.tail_slices > kMaxTailWorkgroups || tiles > kMaxSliceGroups)
      return hipErrorInvalidValue;
    tail_blocks = (int)tiles * a.tail_slices;
  }
  hipLaunchKernelGGL((layer_kernel<BF16, DELTA, MB, NW, NT, KS, RING, TAIL>), dim3(a.main_blocks + tail_blocks),
                     dim3(64 * NW * KS), lds_bytes, stream, a);
  return hipGetLastError();
}

// Workgroups of this instantiation that fit on one compute unit (cached).
template <bool BF16, bool DELTA, int MB, int NW, int KS>
int wgs_per_cu_inst() {
  static const int cached = [] {
    constexpr int lds_bytes = Lds<BF16, DELTA, MB, NW>::TOTAL * KS;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void*>(&layer_kernel<BF16, DELTA, MB, NW, false, KS>),
                                                     64 * NW * KS, lds_bytes) != hipSuccess || n < 1)
      n = 1;
    return n;
  }();
  return cached;
}

// Waves that share one feature tile and split K: four, or two where four private LDS layouts do not
// fit into the 160 KB of a compute unit (0: the layout is single-buffered or too large even twice).
template <bool BF16, bool DELTA, int MB>
constexpr int split_k_waves() {
  using L = Lds<BF16, DELTA, MB, 1>;
  if (!L::DBUF) return 0;
  return L::TOTAL * 4 <= 160 * 1024 ? 4 : L::TOTAL * 2 <= 160 * 1024 ? 2 : 0;
}

// k_waves > 1: the one-wave-tile instantiation whose workgroups split K over that many waves
template <bool BF16, bool DELTA, int MB>
int wgs_per_cu_nw(int NW, int k_waves) {
  if (NW == 8) return wgs_per_cu_inst<BF16, DELTA, MB, 8, 1>();
  if (NW == 4) return wgs_per_cu_inst<BF16, DELTA, MB, 4, 1>();
  constexpr int KS = split_k_waves<BF16, DELTA, MB>();
  if constexpr (KS > 1) {
    if (k_waves == KS) return wgs_per_cu_inst<BF16, DELTA, MB, 1, KS>();
  }
  return wgs_per_cu_inst<BF16, DELTA, MB, 1, 1>();
}

// Streaming loads are used when every row segment a load instruction covers
// starts on a 128-byte line: base pointers, row pitch, block offset and row
// length of every job in the launch are multiples of 128 bytes.
bool job_lines_aligned(const LayerJob& j) { return j.w_off % 32 == 0 && j.K % 32 == 0; }
bool launch_lines_aligned(const LayerArgs& a) {
  bool ok = true;
  if (a.n_cand > 0) ok = ok && reinterpret_cast<uintptr_t>(a.G) % 128 == 0 && a.ldg % 32 == 0 && job_lines_aligned(a.cj);
  if (a.has_base) ok = ok && reinterpret_cast<uintptr_t>(a.x) % 128 == 0 && job_lines_aligned(a.bj);
  return ok;
}

// The shifted column grid serves rows that start 16-byte aligned but not on a line, all of them the same
// distance past one: row lengths that are multiples of 64 columns, 16-byte aligned bases, pitches and blocks.
// Returns 1 for that case, 2 where bases, pitches and blocks are only 8-byte aligned (d mod 4 = 2: every other row of
// a dense G[m x d]; the staging then writes column pairs), 0 where neither holds.
int launch_ring_kind(const LayerArgs& a) {
  if (!a.has_base && a.n_cand <= 0) return 0;
  auto kind = [](uintptr_t base, long long pitch, const LayerJob& j) {
    if (j.K % 64 != 0) return 0;
    if (base % 16 == 0 && pitch % 4 == 0 && j.w_off % 4 == 0) return 1;
    if (base % 8 == 0 && pitch % 2 == 0 && j.w_off % 2 == 0) return 2;
    return 0;
  };
  int k = 1;
  if (a.n_cand > 0) {
    const int kc = kind(reinterpret_cast<uintptr_t>(a.G), a.ldg, a.cj);
    if (kc == 0) return 0;
    if (kc > k) k = kc;
  }
  if (a.has_base) {
    const int kb = kind(reinterpret_cast<uintptr_t>(a.x), 0, a.bj);
    if (kb == 0) return 0;
    if (kb > k) k = kb;
  }
  return k;
}

template <bool BF16, bool DELTA, int MB, int NW>
hipError_t launch_nt(const LayerArgs& a, hipStream_t stream, LaunchShape* shape) {
  // One-tile workgroups whose plan splits K over the waves of a workgroup (every K of the launch gives each
  // wave at least two chunks: the planner's condition, checked again because a wave without chunks would
  // start a copy beyond the operand)
  constexpr int KS = split_k_waves<BF16, DELTA, MB>();
  if constexpr (NW == 1 && KS > 1) {
    if (a.k_waves == KS) {
      const int slices = a.k_slices > 1 ? a.k_slices : 1;
      const bool base_ok = !a.has_base || (a.bj.Kp >> 6) >= 2 * KS * slices;
      const bool cand_ok = a.n_cand == 0 || (a.cj.Kp >> 6) >= 2 * KS * slices;
      if (!((a.has_base || a.n_cand > 0) && base_ok && cand_ok)) return hipErrorInvalidValue;
      if (launch_lines_aligned(a)) return launch_inst<BF16, DELTA, MB, NW, true, KS>(a, stream, shape);
      return launch_inst<BF16, DELTA, MB, NW, false, KS>(a, stream, shape);
    }
  }
  if (NW == 1 && a.k_slices > 1) {
    const bool base_ok = !a.has_base || (a.bj.Kp >> 6) >= 2 * a.k_slices;
    const bool cand_ok = a.n_cand == 0 || (a.cj.Kp >> 6) >= 2 * a.k_slices;
    if (!(base_ok && cand_ok)) return hipErrorInvalidValue;
  }
  if constexpr (NW == 8 && Lds<BF16, DELTA, MB, NW>::DBUF) {
    if (a.tail_slices >= 2) {
      if (launch_lines_aligned(a)) return launch_inst<BF16, DELTA, MB, NW, true, 1, 0, true>(a, stream, shape);
      if constexpr (BF16 && Lds<BF16, DELTA, MB, NW, 1>::DBUF) {
        const int ring = launch_ring_kind(a);
        if (ring == 1) return launch_inst<BF16, DELTA, MB, NW, true, 1, 1, true>(a, stream, shape);
        if (ring == 2) return launch_inst<BF16, DELTA, MB, NW, true, 1, 2, true>(a, stream, shape);
      }
      return launch_inst<BF16, DELTA, MB, NW, false, 1, 0, true>(a, stream, shape);
    }
  }
  if (a.tail_slices >= 2) return hipErrorInvalidValue;   // planned for a launch shape that has no sliced tail
  if (launch_lines_aligned(a)) return launch_inst<BF16, DELTA, MB, NW, true>(a, stream, shape);
  if constexpr (BF16 && NW > 1 && Lds<BF16, DELTA, MB, NW, 1>::DBUF) {
    const int ring = launch_ring_kind(a);
    if (ring == 1) return launch_inst<BF16, DELTA, MB, NW, true, 1, 1>(a, stream, shape);
    if (ring == 2) return launch_inst<BF16, DELTA, MB, NW, true, 1, 2>(a, stream, shape);
  }
  return launch_inst<BF16, DELTA, MB, NW, false>(a, stream, shape);
}

template <bool BF16, bool DELTA, int MB>
hipError_t launch_nw(const LayerArgs& a, int NW, hipStream_t stream, LaunchShape* shape) {
  if (NW == 8) return launch_nt<BF16, DELTA, MB, 8>(a, stream, shape);
  if (NW == 4) return launch_nt<BF16, DELTA, MB, 4>(a, stream, shape);
  return launch_nt<BF16, DELTA, MB, 1>(a, stream, shape);
}

// Waves per workgroup (32 output features each): the widest workgroup that still
// gives every compute unit work, since a wider workgroup re-reads less of the
// activations per byte of weights; narrow layers fall back to one wave to spread
// over more compute units.
int pick_nw(int rows, int n_src) {
  if ((long long)((rows + 255) / 256) * n_src >= 256) return 8;
  if ((long long)((rows + 127) / 128) * n_src >= 256) return 4;
  return 1;
}

// Waves per workgroup of a launch, from the job that dominates it.
int launch_nw_for(const LayerArgs& a) {
  if (a.n_cand > 0) return pick_nw(cover_rows(a.cj.N, a.cj.last), a.n_cand);
  return pick_nw(cover_rows(a.bj.N, a.bj.last), 1);
}

}  // namespace

}  // namespace zeno

// The kernel is compiled in twelve objects so that the instantiations build in parallel: four source files, one per
// (operand type, second product) pair, each compiled once per number of row blocks (-DZENO_LAYER_MB=1, 2, 4; without
// the definition a file holds all three).  Each object defines the two entry points of its (pair, row blocks) that the
// dispatcher in zeno_layer.hip calls.
#define ZENO_LAYER_INSTANCE_MB_(NAME, BF16, DELTA, MB)                                                       \
  namespace zeno {                                                                                           \
  hipError_t launch_layer_##NAME##_mb##MB(const LayerArgs& a, int NW, hipStream_t stream, LaunchShape* shape) { \
    return launch_nw<BF16, DELTA, MB>(a, NW, stream, shape);                                                 \
  }                                                                                                          \
  int wgs_per_cu_##NAME##_mb##MB(int NW, int k_waves) { return wgs_per_cu_nw<BF16, DELTA, MB>(NW, k_waves); }   \
  }
#define ZENO_LAYER_INSTANCE_MB(NAME, BF16, DELTA, MB) ZENO_LAYER_INSTANCE_MB_(NAME, BF16, DELTA, MB)
#ifdef ZENO_LAYER_MB
#define ZENO_LAYER_INSTANCE(NAME, BF16, DELTA) ZENO_LAYER_INSTANCE_MB(NAME, BF16, DELTA, ZENO_LAYER_MB)
#else
#define ZENO_LAYER_INSTANCE(NAME, BF16, DELTA) \
  ZENO_LAYER_INSTANCE_MB(NAME, BF16, DELTA, 1) \
  ZENO_LAYER_INSTANCE_MB(NAME, BF16, DELTA, 2) \
  ZENO_LAYER_INSTANCE_MB(NAME, BF16, DELTA, 4)
#endif

#endif  // ZENO_LAYER_IMPL_H_
