// Internal declarations shared by the translation units of the Zeno HIP library.
// Nothing here is part of the C ABI (that is include/zeno.h).
#ifndef ZENO_INTERNAL_H_
#define ZENO_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zeno.h"

// Host-side model object behind zeno_model_t: a chain of linear layers (kind 0) or a
// convolutional network (kind 1: 3 x 3 convolutions, then one fully connected layer).
struct zeno_model {
  int kind;
  zeno_model_desc_t desc;          // kind 0; for kind 1 it describes the fully connected layer alone
  int64_t w_off[ZENO_MAX_LAYERS];  // offset of W_l (l = 0..L-1) inside a parameter vector
  int64_t b_off[ZENO_MAX_LAYERS];  // offset of b_l, or -1
  int64_t d;
  // kind 1
  zeno_cnn_desc_t cnn;
  int map_h[ZENO_MAX_CONV + 1], map_w[ZENO_MAX_CONV + 1], map_c[ZENO_MAX_CONV + 1];  // input and every map
  int64_t conv_w_off[ZENO_MAX_CONV], conv_b_off[ZENO_MAX_CONV];
};

namespace zeno {

// Four floats with 4-byte alignment: rows of G and the per-layer blocks inside a
// row start at arbitrary 4-byte offsets, and gfx950 global loads/stores of 128
// bits only need dword alignment.
struct __attribute__((packed, aligned(4))) f4u {
  float x, y, z, w;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef f32x4 f32x4_a4 __attribute__((aligned(4)));  // same, for 4-byte aligned addresses

// Streaming (non-temporal) 128-bit load from a 4-byte aligned address: rows of G
// are read exactly once, so they should not displace reusable lines in the caches.
__device__ inline f32x4 load_stream4(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(p));
}
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// One linear layer as a launch of the streaming layer kernel sees it.
struct LayerJob {
  long long w_off;     // offset of W_l inside a parameter vector
  long long b_off;     // offset of b_l, or -1
  int N, K;            // layer width out / in
  int Kp;              // K rounded up to a multiple of 64 (tiled operand width)
  int Np;              // N rounded up to a multiple of 64 (tiled width of the next layer's operand)
  int last;            // 1: output layer (raw fp32 results instead of tiled activations)
  const void* A_base;  // tiled activations of the pass at x that feed this layer
  void* Wt;            // W_l in matrix-operand order (written by the pass at x, read by the candidates); may be NULL
  float* Z0;           // [n_r x N] pre-activations at x (written by the pass at x, read by the candidates)
  void* H_base;        // tiled output activations of the pass at x (hidden layers)
};

// One launch of the streaming layer kernel (zeno_layer.hip): the candidates'
// pass through layer `cj` (n_cand workgroup columns, may be 0) and, in the same
// launch, the pass at x through layer `bj` (has_base; normally the NEXT layer,
// whose input the previous launch finished), so that the short pass at x hides
// behind the long candidate stream.
struct LayerArgs {
  const float* G;       // [m x d]
  const float* x;       // [d]
  long long ldg;        // floats between consecutive rows of G
  int n_cand;           // candidates in this launch (0 or m)
  int has_base;         // 1: the launch also runs the pass at x through bj
  int base_blocks;      // leading block indices reserved for the pass at x (multiple of 8)
  int n_r;              // valid samples (rows) in this pass
  LayerJob cj, bj;
  const void* D_cand;   // tiled scaled activation differences of candidate 0 (delta launches only)
  long long A_stride;   // bytes between consecutive candidates in D_cand
  float* dZ;            // [m x n_r x N] change of the output layer's pre-activations (last layer)
  void* Dl_cand;        // tiled scaled output differences of candidate 0 (hidden layers)
  long long H_stride;   // bytes between consecutive candidates in Dl_cand
  float gamma;
  float neg_inv_gamma;  // -1/gamma, or 0 when gamma == 0
  double* norm_partials;  // [m x P] partial sums of squares, or NULL in passes after the first
  // K split of a launch of one-wave tiles (the launcher fills these in from layer_k_plan): k_waves waves of a
  // workgroup share a feature tile and split K (1, or the widest split the LDS layout allows), and K is also
  // split over k_slices workgroups per tile.  Each of those writes its partial accumulators to slice_partials,
  // and the last one to arrive (slice_counters, zero on entry, zero again on exit) adds them in slice order and
  // finishes the tile.  Tiles are numbered [pass at x: its feature tiles] [candidates: slice_group0 +
  // candidate x tiles + tile].
  int k_waves;
  int k_slices;
  long long slice_group0;
  float* slice_partials;
  unsigned int* slice_counters;
  int P;                // partial slots per candidate
  int p_off;            // first slot of this layer
  // Sliced tail of a launch of eight-wave workgroups (see layer_tail_slices): the tiles of the last tail_cand
  // candidates, and of the pass at x if the launch carries it, run as tail_slices K slices each, in the blocks
  // from main_blocks on.  Their partial accumulators go through slice_partials / slice_counters as well; their
  // partial norms to the slots tail_p_off + tile * tail_slices + slice.
  int tail_cand;
  int tail_slices;
  int tail_p_off;
  int main_blocks;      // filled in by the launcher
};

// Launchers.  Each returns the hipError_t of its launches.
// also clears the n_counters workgroup-arrival counters of the pass (may be 0)
// ... and n_zero doubles at `zero` (the candidates' partial-norm slots; may be 0)
hipError_t launch_pack_features(const float* features, int n_r, int K, int Kp, int MB, bool bf16,
                                void* tiled, unsigned int* counters, int n_counters, double* zero, long long n_zero,
                                hipStream_t stream);
// Limits of a launch whose K is split over workgroups: bytes of partial accumulators (tiles x slices x row
// blocks x 4 KB) and tiles (= arrival counters).  One buffer of each serves all launches of a pass, which run
// one after the other and leave the counters at zero.
constexpr size_t kSlicePartialBytes = size_t(8) << 20;
constexpr int kMaxSliceGroups = 2048;
// Sliced tails: at most this many eight-wave workgroups (tiles x slices), each handing over 8 x row blocks x 4 KB
constexpr int kMaxTailWorkgroups = 256;
inline size_t tail_partial_bytes(int MB) { return (size_t)kMaxTailWorkgroups * 8 * MB * 16 * 64 * sizeof(float); }
struct KPlan {
  int k_waves;    // waves of a workgroup that share a feature tile and split K
  int k_slices;   // workgroups per feature tile
};
// The K split a launch with NW waves per workgroup takes (NW > 1: none).  device = false: no device is asked
// for occupancies and the result is the widest split any device could be given (for sizing and checking).
KPlan layer_k_plan(const LayerArgs& a, bool bf16, bool delta, int MB, int NW, bool device);
// Which instantiation of the layer kernel a launch took (reported in the per-launch timing records).
struct LaunchShape {
  int waves;       // waves per workgroup that own different feature tiles (1, 4 or 8)
  int k_split;     // waves that share one feature tile and split K (1, 2 or 4)
  int k_slices;    // workgroups that share one feature tile and split K (1 to 8)
  int streaming;   // 1: rows read with non-temporal loads (line-aligned layout), 2: the same on the shifted column grid
  int row_blocks;  // 32-sample accumulator blocks per wave (1, 2 or 4)
};
hipError_t launch_layer(const LayerArgs& a, bool bf16, bool delta, int MB, hipStream_t stream,
                        LaunchShape* shape = nullptr);
bool layer_merge_pays(const LayerArgs& a, bool bf16, bool delta, int MB);  // run a.bj inside the candidates' launch?
// K slices for the tiles of the last (n_cand - *n_main) candidates of an eight-wave launch, or 0: no sliced tail
int layer_tail_slices(const LayerArgs& a, bool bf16, bool delta, int MB, int* n_main);
int layer_tiles(const LayerArgs& a, bool bf16, bool delta, int MB);   // partial-norm slots per candidate the launch fills
int layer_nw(const LayerArgs& a, bool bf16, bool delta, int MB);     // waves per workgroup the launch will use
// Extents a launch with NW waves per workgroup writes (bytes / floats / slots, counted from the start of each buffer).
struct LayerExtents {
  long long wt_bytes;          // operand-order copy of W (pass at x)
  long long hbase_bytes;       // tiled activations of the pass at x
  long long z0_floats;         // pre-activations at x
  long long d_bytes_per_cand;  // tiled scaled activation differences of one candidate
  long long dz_floats;         // output layer's change of pre-activations, all candidates
  int norm_slots;              // partial-norm slots per candidate
  long long slice_bytes;       // partial accumulators of a launch with K split over workgroups
  int slice_counters;          // arrival counters it uses
};
LayerExtents layer_extents(const LayerArgs& a, bool bf16, bool delta, int MB, int NW, bool device);
hipError_t launch_loss(const float* Z0, const float* dZ, const int32_t* labels, const float* targets,
                       int loss, int m, int n_r_total, int chunk_begin, int chunk_rows, int C,
                       double* sample_diff, hipStream_t stream);
hipError_t launch_score_combine(const double* sample_diff, const double* norm_partials, int P, int m,
                                int n_r_total, float rho, float* scores, hipStream_t stream);
// the same with the candidates' partial norms P_stride slots apart, the first P of them in use
hipError_t launch_score_combine_strided(const double* sample_diff, const double* norm_partials, int P_stride, int P,
                                        int m, int n_r_total, float rho, float* scores, hipStream_t stream);
// x_next != nullptr: also write x_next = x - gamma * average (out may then be nullptr)
hipError_t launch_masked_average(const float* G, long long ldg, const float* scores, int m, long long d, int b,
                                 float* out, int32_t* selected, hipStream_t stream, float gamma = 0.f,
                                 const float* x = nullptr, float* x_next = nullptr);
size_t krum_workspace_bytes(int m);
hipError_t launch_krum(const float* G, long long ldg, int m, long long d, int b, float* out, int32_t* chosen,
                       float* scores_out, void* workspace, hipStream_t stream);
hipError_t launch_median(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream);          // m <= 128
hipError_t launch_median_select(const float* G, long long ldg, int m, long long d, float* out, hipStream_t stream);   // m <= 1024

// ---- convolutional models (zeno_conv.hip)
// One 3 x 3 convolution (zero padding 1) as the kernel sees it.
struct ConvLayer {
  long long w_off, b_off;  // offsets inside a parameter vector; b_off = -1: no bias
  int Hin, Win, Cin, Hout, Wout, Cout, stride;
};
struct ConvArgs {
  const float* G;         // [m x d]
  const float* x;         // [d]
  long long ldg;
  int n_cand;             // m: the candidates' pass; 0: the pass at x
  int n_r;
  ConvLayer L;
  const float* H0_in;     // input map of the pass at x, NHWC [n_r * Hin * Win x Cin] (the images for the first convolution)
  const float* D_in;      // candidate 0's scaled change of the input map, or nullptr (first convolution)
  long long D_in_stride;  // floats between candidates
  float* Z0;              // [rows x Cout] pre-activations at x: written by the pass at x, read by the candidates
  float* out;             // pass at x: relu map; candidates: candidate 0's scaled change of the output map
  long long out_stride;   // floats between candidates (candidates' pass)
  int tiled_out;          // 1: out is the operand of the fully connected layer: rows = samples, k = (position, channel),
  int Kp_fc;              //    in matrix-operand order of padded width Kp_fc
  float gamma, neg_inv_gamma;
};
hipError_t launch_conv(const ConvArgs& a, hipStream_t stream);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);
// sum of squares of G[s][begin .. begin+count) for every candidate, in n_blocks fixed pieces -> partials[s*P + p_off + blk]
hipError_t launch_sumsq(const float* G, long long ldg, int m, long long begin, long long count, int n_blocks,
                        double* partials, int P, int p_off, hipStream_t stream);

}  // namespace zeno
#endif
