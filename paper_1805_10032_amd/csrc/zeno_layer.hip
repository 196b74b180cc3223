// Dispatcher of the streaming layer kernel: launch shapes, the choice between merged
// and separate launches of the pass at x, and the packing of the batch.  The kernel
// itself lives in zeno_layer_impl.h and is compiled in twelve objects (the four files
// zeno_layer_{bf16,f32}_{first,delta}.hip, each once per number of row blocks).
#include <cstring>

#include "zeno_layer_impl.h"

namespace zeno {

// the entry points of the twelve kernel objects: (operand type, second product) x row blocks
#define ZENO_DECLARE_LAYER(NAME)                                                                                  \
  hipError_t launch_layer_##NAME##_mb1(const LayerArgs& a, int NW, hipStream_t stream, LaunchShape* shape);       \
  hipError_t launch_layer_##NAME##_mb2(const LayerArgs& a, int NW, hipStream_t stream, LaunchShape* shape);       \
  hipError_t launch_layer_##NAME##_mb4(const LayerArgs& a, int NW, hipStream_t stream, LaunchShape* shape);       \
  int wgs_per_cu_##NAME##_mb1(int NW, int k_waves);                                                               \
  int wgs_per_cu_##NAME##_mb2(int NW, int k_waves);                                                               \
  int wgs_per_cu_##NAME##_mb4(int NW, int k_waves);                                                               \
  static hipError_t launch_layer_##NAME(const LayerArgs& a, int MB, int NW, hipStream_t stream, LaunchShape* shape) { \
    return MB == 1 ? launch_layer_##NAME##_mb1(a, NW, stream, shape)                                              \
         : MB == 2 ? launch_layer_##NAME##_mb2(a, NW, stream, shape)                                              \
                   : launch_layer_##NAME##_mb4(a, NW, stream, shape);                                             \
  }                                                                                                               \
  static int wgs_per_cu_##NAME(int MB, int NW, int k_waves) {                                                     \
    return MB == 1 ? wgs_per_cu_##NAME##_mb1(NW, k_waves) : MB == 2 ? wgs_per_cu_##NAME##_mb2(NW, k_waves)        \
                                                                     : wgs_per_cu_##NAME##_mb4(NW, k_waves);      \
  }
ZENO_DECLARE_LAYER(bf16_delta)
ZENO_DECLARE_LAYER(bf16_first)
ZENO_DECLARE_LAYER(f32_delta)
ZENO_DECLARE_LAYER(f32_first)
#undef ZENO_DECLARE_LAYER

template <bool BF16, bool DELTA>
static int ks_waves_for(int MB) {
  return MB == 1 ? split_k_waves<BF16, DELTA, 1>() : MB == 2 ? split_k_waves<BF16, DELTA, 2>() : split_k_waves<BF16, DELTA, 4>();
}

static int compute_units() {
  static const int n_cu = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
      v = 256;
    return v;
  }();
  return n_cu;
}

static int wgs_per_cu(bool bf16, bool delta, int MB, int NW, int k_waves = 1) {
  return bf16 ? (delta ? wgs_per_cu_bf16_delta(MB, NW, k_waves) : wgs_per_cu_bf16_first(MB, NW, k_waves))
              : (delta ? wgs_per_cu_f32_delta(MB, NW, k_waves) : wgs_per_cu_f32_first(MB, NW, k_waves));
}

static int ks_waves(bool bf16, bool delta, int MB) {
  return bf16 ? (delta ? ks_waves_for<true, true>(MB) : ks_waves_for<true, false>(MB))
              : (delta ? ks_waves_for<false, true>(MB) : ks_waves_for<false, false>(MB));
}

// Waves per workgroup of a launch.  Where eight would be picked, four are taken instead if two
// such workgroups fit on a compute unit and the eight-wave workgroups do not fill their rounds of
// (compute units x resident workgroups) almost exactly: the eight waves of a workgroup that has a
// compute unit to itself all wait at the same barrier once per chunk, while two four-wave
// workgroups run out of step and fill each other's waits (workload 4: 800 eight-wave workgroups
// are 3.1 rounds, four waves gain 2-4 % per layer; workload 5: 1024 are exactly four rounds and
// eight waves, which copy the activations once per 256 features instead of once per 128, win).
static int nw_for(const LayerArgs& a, bool bf16, bool delta, int MB) {
  if (a.tail_slices >= 2) return 8;   // planned with a sliced tail, which exists for eight-wave workgroups
  const int nw = launch_nw_for(a);
  if (nw != 8 || a.n_cand <= 0) return nw;
  if (wgs_per_cu(bf16, delta, MB, 4) < 2) return 8;
  const long long slots = (long long)compute_units() * wgs_per_cu(bf16, delta, MB, 8);
  const long long wgs = (long long)job_tiles(a.cj, 256) * a.n_cand;
  const long long rounds = (wgs + slots - 1) / slots;
  return 10 * wgs >= 9 * rounds * slots ? 8 : 4;
}

int layer_nw(const LayerArgs& a, bool bf16, bool delta, int MB) { return nw_for(a, bf16, delta, MB); }

// K split of a launch of one-wave tiles.  Such a launch has few feature tiles (the pass at x: N/32; a narrow
// layer: one or a few per candidate), so a tile's K is divided among the k_waves waves of its workgroup (which
// add their accumulators through LDS) and among k_slices workgroups (which add theirs through memory, the
// last one to arrive finishing the tile).  Every wave keeps at least two chunks.
//  * The waves of a workgroup split K as widely as the LDS layout allows (four or two private copies).
//  * Workgroups per tile: as many as bring the launch to about one workgroup per compute unit, at most 8.
//    Measured: on an otherwise idle chip every doubling helps down to two chunks per wave (a ten-class
//    layer behind 4096 inputs, 20 candidates: 8 slices 35 us, 4 slices 42 us), while a launch that already
//    has a workgroup per compute unit only gets slower (its workgroups queue, and the round trips of the
//    hand-over, cheap on an idle chip, take several microseconds each once the memory system is loaded).
//  * One exception: a launch with somewhat more tiles than compute units whose wide workgroups fit only one
//    per compute unit (four LDS layouts) would run a full round and a nearly empty one.  One-wave
//    workgroups, two per tile, several per compute unit, run it in one round (3072 -> 512, 20 candidates:
//    54 -> 48 us; three or four per tile: 53, 64 us).
KPlan layer_k_plan(const LayerArgs& a, bool bf16, bool delta, int MB, int NW, bool device) {
  KPlan plan = {1, 1};
  if (NW != 1 || (!a.has_base && a.n_cand <= 0)) return plan;
  const int base_chunks = a.has_base ? a.bj.Kp >> 6 : 1 << 30, cand_chunks = a.n_cand > 0 ? a.cj.Kp >> 6 : 1 << 30;
  const int min_chunks = base_chunks < cand_chunks ? base_chunks : cand_chunks;
  const long long groups = (a.has_base ? job_tiles(a.bj, 32) : 0) + (long long)(a.n_cand > 0 ? job_tiles(a.cj, 32) : 0) * a.n_cand;
  const int ks_max = ks_waves(bf16, delta, MB);
  const bool wide_ok = ks_max > 1 && min_chunks >= 2 * ks_max;
  const bool can_slice = a.slice_partials != nullptr && a.slice_counters != nullptr && groups <= kMaxSliceGroups;
  // most workgroups per tile that the buffers and the two-chunk rule allow
  auto max_slices = [&](int kw) {
    if (!can_slice) return 1;
    long long s = min_chunks / (2 * kw);
    const long long by_bytes = (long long)(kSlicePartialBytes / ((size_t)MB * 16 * 64 * sizeof(float))) / groups;
    if (s > by_bytes) s = by_bytes;
    if (s > 8) s = 8;
    return s < 1 ? 1 : (int)s;
  };
  plan.k_waves = wide_ok ? ks_max : 1;
  if (!device) {
    // sizing: the split over workgroups is widest for one-wave workgroups
    plan.k_slices = max_slices(1);
    return plan;
  }
  const int n_cu = compute_units();
  long long s = n_cu / groups;
  const int cap = max_slices(plan.k_waves);
  if (s > cap) s = cap;
  plan.k_slices = s < 1 ? 1 : (int)s;
  if (wide_ok && plan.k_slices == 1 && max_slices(1) >= 2 && (a.n_cand > 0 ? cand_chunks : base_chunks) >= 32 &&
      groups > (long long)n_cu * wgs_per_cu(bf16, delta, MB, 1, ks_max) && 2 * groups <= 3LL * n_cu &&
      2 * groups <= (long long)n_cu * wgs_per_cu(bf16, delta, MB, 1, 1)) {
    plan.k_waves = 1;
    plan.k_slices = 2;
  }
  return plan;
}

// What a launch of workgroup width NW writes, from the kernel's own index formulas: the
// host checks these against the workspace slots before anything is enqueued.
LayerExtents layer_extents(const LayerArgs& a, bool bf16, bool delta, int MB, int NW, bool device) {
  LayerExtents e;
  std::memset(&e, 0, sizeof(e));
  const int esize = bf16 ? 2 : 4, wregs = bf16 ? 4 : 8, n_pad = 32 * MB;
  auto tiled_bytes = [&](int Np) {
    const long long last = bf16 ? tiled_index<true>(n_pad - 1, Np - 1, Np) : tiled_index<false>(n_pad - 1, Np - 1, Np);
    return (last + 1) * esize;
  };
  if (a.has_base) {
    const LayerJob& j = a.bj;
    // every wave of every workgroup of the pass at x stores its 32-row tile of W, chunk by chunk
    if (j.Wt != nullptr) e.wt_bytes = (long long)job_tiles(j, 32 * NW) * NW * (j.Kp >> 6) * wregs * 1024;
    e.z0_floats = (long long)a.n_r * j.N;
    if (!j.last) e.hbase_bytes = tiled_bytes(j.Np);
  }
  if (a.n_cand > 0) {
    const LayerJob& j = a.cj;
    if (j.last) e.dz_floats = (long long)a.n_cand * a.n_r * j.N;
    else e.d_bytes_per_cand = tiled_bytes(j.Np);
    e.norm_slots = job_tiles(j, 32 * NW);
  }
  // K split over workgroups as well (one-wave tiles)
  const KPlan kp = layer_k_plan(a, bf16, delta, MB, NW, device);
  if (kp.k_slices > 1) {
    const long long groups = (a.has_base ? job_tiles(a.bj, 32) : 0) + (long long)(a.n_cand > 0 ? job_tiles(a.cj, 32) : 0) * a.n_cand;
    e.slice_bytes = groups * kp.k_slices * MB * 16 * 64 * (long long)sizeof(float);
    e.slice_counters = (int)groups;
    if (a.n_cand > 0) e.norm_slots *= kp.k_slices;
  }
  if (a.tail_slices >= 2 && NW == 8) {
    const long long tiles = (a.has_base ? job_tiles(a.bj, 256) : 0) + (long long)job_tiles(a.cj, 256) * a.tail_cand;
    e.slice_bytes = tiles * a.tail_slices * 8 * MB * 16 * 64 * (long long)sizeof(float);
    e.slice_counters = (int)tiles;
    e.norm_slots = a.tail_p_off - a.p_off + job_tiles(a.cj, 256) * a.tail_slices;   // both ranges, counted from p_off
  }
  return e;
}

// Does the eight-wave workgroup of this kind double-buffer its activation chunks (the sliced tail needs it)?
static bool wide_double_buffered(bool bf16, bool delta, int MB) {
  auto pick = [&](auto mb) {
    constexpr int M = decltype(mb)::value;
    return bf16 ? (delta ? Lds<true, true, M, 8>::DBUF : Lds<true, false, M, 8>::DBUF)
                : (delta ? Lds<false, true, M, 8>::DBUF : Lds<false, false, M, 8>::DBUF);
  };
  return MB == 1 ? pick(std::integral_constant<int, 1>{}) : MB == 2 ? pick(std::integral_constant<int, 2>{})
                                                                     : pick(std::integral_constant<int, 4>{});
}

// Sliced tail of a candidate launch of eight-wave workgroups.  When the workgroups of the launch do not fill their
// last round of resident slots, the candidates of that round (and the pass at x, if the launch carries it) are cut
// into K slices, as many as bring their workgroups to about one round: the round then lasts a fraction of a whole
// tile's time, and the slices start as soon as slots free up behind the whole tiles.  Workload 4's 2048-wide layers
// (100 candidates x 8 tiles = 3.125 rounds of 256): candidates 96..99 and the pass at x are 40 tiles, cut six ways.
// Not where the workgroup is single-buffered.
int layer_tail_slices(const LayerArgs& a, bool bf16, bool delta, int MB, int* n_main_out) {
  *n_main_out = a.n_cand;
  if (a.n_cand <= 0 || launch_nw_for(a) != 8 || a.slice_partials == nullptr || a.slice_counters == nullptr) return 0;
  if (!wide_double_buffered(bf16, delta, MB)) return 0;
  const long long slots = (long long)compute_units() * wgs_per_cu(bf16, delta, MB, 8);
  const int tiles8 = job_tiles(a.cj, 256);
  const long long full = (long long)tiles8 * a.n_cand / slots * slots;
  const int n_main = (int)(full / tiles8), rest = a.n_cand - n_main;
  // (candidates that fill their rounds exactly leave the pass at x to a launch of its own: as a sliced tail of 16
  // tiles x 8 slices behind workload 5's 4096-wide layers it took 60 us, twice what the launch of one-wave tiles
  // with K split over waves and workgroups takes; with four row blocks the hand-over alone is seven round trips)
  if (n_main <= 0 || rest <= 0 || full % tiles8 != 0) return 0;
  const long long tail_tiles = (long long)rest * tiles8 + (a.has_base ? job_tiles(a.bj, 256) : 0);
  int min_chunks = a.cj.Kp >> 6;
  if (a.has_base && (a.bj.Kp >> 6) < min_chunks) min_chunks = a.bj.Kp >> 6;
  long long S = slots / tail_tiles;
  if (S > kMaxTailWorkgroups / tail_tiles) S = kMaxTailWorkgroups / tail_tiles;
  if (S > min_chunks / 4) S = min_chunks / 4;
  if (S > 8) S = 8;
  if (S < 2) return 0;
  *n_main_out = n_main;
  return (int)S;
}

int layer_tiles(const LayerArgs& a, bool bf16, bool delta, int MB) {
  const int NW = nw_for(a, bf16, delta, MB);
  const int tail = a.tail_slices >= 2 ? job_tiles(a.cj, 256) * a.tail_slices : 0;
  return job_tiles(a.cj, 32 * NW) * layer_k_plan(a, bf16, delta, MB, NW, true).k_slices + tail;
}

// Should the pass at x (a.bj) ride in the candidates' launch?  Workgroups run in
// rounds of (compute units x resident workgroups); the extra workgroups are free
// when they fit into the last round and cost a whole extra round when the
// candidates fill their rounds exactly, unless there are many rounds anyway.
bool layer_merge_pays(const LayerArgs& a, bool bf16, bool delta, int MB) {
  if (a.n_cand <= 0) return true;
  const int n_cu = compute_units();
  const int NW = nw_for(a, bf16, delta, MB);
  const int per_cu = wgs_per_cu(bf16, delta, MB, NW);
  const long long slots = (long long)n_cu * per_cu;
  const long long cand = (long long)job_tiles(a.cj, 32 * NW) * a.n_cand;
  const long long base = job_tiles(a.bj, 32 * NW);
  const long long rounds_without = (cand + slots - 1) / slots, rounds_with = (cand + base + slots - 1) / slots;
  return rounds_with == rounds_without || rounds_without >= 8;
}

hipError_t launch_pack_features(const float* features, int n_r, int K, int Kp, int MB, bool bf16, void* tiled,
                                unsigned int* counters, int n_counters, double* zero, long long n_zero,
                                hipStream_t stream) {
  const int n_pad = 32 * MB;
  const long long total = (long long)n_pad * Kp;
  const int grid = (int)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
  if (bf16) {
    hipLaunchKernelGGL(pack_features_kernel<true>, dim3(grid), dim3(256), 0, stream, features, n_r, K, Kp, n_pad, tiled,
                       counters, n_counters, zero, n_zero);
  } else {
    hipLaunchKernelGGL(pack_features_kernel<false>, dim3(grid), dim3(256), 0, stream, features, n_r, K, Kp, n_pad, tiled,
                       counters, n_counters, zero, n_zero);
  }
  return hipGetLastError();
}

hipError_t launch_layer(const LayerArgs& a, bool bf16, bool delta, int MB, hipStream_t stream, LaunchShape* shape) {
  const int NW = nw_for(a, bf16, delta, MB);
  LayerArgs b = a;
  const KPlan kp = layer_k_plan(a, bf16, delta, MB, NW, true);
  b.k_waves = kp.k_waves;
  b.k_slices = kp.k_slices;
  b.slice_group0 = (a.has_base && a.n_cand > 0) ? job_tiles(a.bj, 32) : 0;
  if (bf16) {
    return delta ? launch_layer_bf16_delta(b, MB, NW, stream, shape) : launch_layer_bf16_first(b, MB, NW, stream, shape);
  }
  return delta ? launch_layer_f32_delta(b, MB, NW, stream, shape) : launch_layer_f32_first(b, MB, NW, stream, shape);
}

}  // namespace zeno
