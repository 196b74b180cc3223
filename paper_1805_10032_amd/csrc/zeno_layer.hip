// Dispatcher of the streaming layer kernel: launch shapes, the choice between merged
// and separate launches of the pass at x, and the packing of the batch.  The kernel
// itself lives in zeno_layer_impl.h and is compiled in four translation units
// (zeno_layer_{bf16,f32}_{first,delta}.hip).
#include <cstring>

#include "zeno_layer_impl.h"

namespace zeno {

hipError_t launch_layer_bf16_delta(const LayerArgs& a, int MB, int NW, hipStream_t stream, LaunchShape* shape);
hipError_t launch_layer_bf16_first(const LayerArgs& a, int MB, int NW, hipStream_t stream, LaunchShape* shape);
hipError_t launch_layer_f32_delta(const LayerArgs& a, int MB, int NW, hipStream_t stream, LaunchShape* shape);
hipError_t launch_layer_f32_first(const LayerArgs& a, int MB, int NW, hipStream_t stream, LaunchShape* shape);
int ks_waves_bf16_delta(int MB);
int ks_waves_bf16_first(int MB);
int ks_waves_f32_delta(int MB);
int ks_waves_f32_first(int MB);
int wgs_per_cu_bf16_delta(int MB, int NW);
int wgs_per_cu_bf16_first(int MB, int NW);
int wgs_per_cu_f32_delta(int MB, int NW);
int wgs_per_cu_f32_first(int MB, int NW);

static int compute_units() {
  static const int n_cu = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
      v = 256;
    return v;
  }();
  return n_cu;
}

static int wgs_per_cu(bool bf16, bool delta, int MB, int NW) {
  return bf16 ? (delta ? wgs_per_cu_bf16_delta(MB, NW) : wgs_per_cu_bf16_first(MB, NW))
              : (delta ? wgs_per_cu_f32_delta(MB, NW) : wgs_per_cu_f32_first(MB, NW));
}

// Waves per workgroup of a launch.  Where eight would be picked, four are taken instead if two
// such workgroups fit on a compute unit and the eight-wave workgroups do not fill their rounds of
// (compute units x resident workgroups) almost exactly: the eight waves of a workgroup that has a
// compute unit to itself all wait at the same barrier once per chunk, while two four-wave
// workgroups run out of step and fill each other's waits (workload 4: 800 eight-wave workgroups
// are 3.1 rounds, four waves gain 2-4 % per layer; workload 5: 1024 are exactly four rounds and
// eight waves, which copy the activations once per 256 features instead of once per 128, win).
static int nw_for(const LayerArgs& a, bool bf16, bool delta, int MB) {
  const int nw = launch_nw_for(a);
  if (nw != 8 || a.n_cand <= 0) return nw;
  if (wgs_per_cu(bf16, delta, MB, 4) < 2) return 8;
  const long long slots = (long long)compute_units() * wgs_per_cu(bf16, delta, MB, 8);
  const long long wgs = (long long)job_tiles(a.cj, 256) * a.n_cand;
  const long long rounds = (wgs + slots - 1) / slots;
  return 10 * wgs >= 9 * rounds * slots ? 8 : 4;
}

int layer_nw(const LayerArgs& a, bool bf16, bool delta, int MB) { return nw_for(a, bf16, delta, MB); }

// K slices (workgroups per tile) the launch will take: the conditions of the launcher in zeno_layer_impl.h.
static int launch_slices(const LayerArgs& a, bool bf16, bool delta, int MB) {
  if (nw_for(a, bf16, delta, MB) != 1) return 1;
  const int KS = bf16 ? (delta ? ks_waves_bf16_delta(MB) : ks_waves_bf16_first(MB))
                      : (delta ? ks_waves_f32_delta(MB) : ks_waves_f32_first(MB));
  if (KS <= 1) return 1;
  const bool base_ok = !a.has_base || (a.bj.Kp >> 6) >= 2 * KS;
  const bool cand_ok = a.n_cand == 0 || (a.cj.Kp >> 6) >= 2 * KS;
  if (!((a.has_base || a.n_cand > 0) && base_ok && cand_ok)) return 1;
  return slices_for(a, KS);
}

// What a launch of workgroup width NW writes, from the kernel's own index formulas: the
// host checks these against the workspace slots before anything is enqueued.
LayerExtents layer_extents(const LayerArgs& a, bool bf16, bool delta, int MB, int NW) {
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
  // K split over workgroups as well (one-wave tiles, the pass at x or the candidates alone)
  if (NW == 1 && a.slice_partials != nullptr && (a.has_base != 0) != (a.n_cand > 0)) {
    const int KS = bf16 ? (delta ? ks_waves_bf16_delta(MB) : ks_waves_bf16_first(MB))
                        : (delta ? ks_waves_f32_delta(MB) : ks_waves_f32_first(MB));
    const bool long_enough = ((a.has_base ? a.bj.Kp : a.cj.Kp) >> 6) >= 2 * KS;
    const int worst = (KS > 1 && long_enough) ? slices_for(a, KS) : 1;
    if (worst > 1) {
      const long long groups = (long long)job_tiles(a.has_base ? a.bj : a.cj, 32) * (a.has_base ? 1 : a.n_cand);
      e.slice_bytes = groups * worst * MB * 16 * 64 * (long long)sizeof(float);
      e.slice_counters = (int)groups;
      if (a.n_cand > 0) e.norm_slots *= worst;
    }
  }
  return e;
}

int layer_tiles(const LayerArgs& a, bool bf16, bool delta, int MB) {
  return job_tiles(a.cj, 32 * nw_for(a, bf16, delta, MB)) * launch_slices(a, bf16, delta, MB);
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
                                unsigned int* counters, int n_counters, hipStream_t stream) {
  const int n_pad = 32 * MB;
  const long long total = (long long)n_pad * Kp;
  const int grid = (int)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
  if (bf16) {
    hipLaunchKernelGGL(pack_features_kernel<true>, dim3(grid), dim3(256), 0, stream, features, n_r, K, Kp, n_pad, tiled,
                       counters, n_counters);
  } else {
    hipLaunchKernelGGL(pack_features_kernel<false>, dim3(grid), dim3(256), 0, stream, features, n_r, K, Kp, n_pad, tiled,
                       counters, n_counters);
  }
  return hipGetLastError();
}

hipError_t launch_layer(const LayerArgs& a, bool bf16, bool delta, int MB, hipStream_t stream, LaunchShape* shape) {
  const int NW = nw_for(a, bf16, delta, MB);
  if (bf16) {
    return delta ? launch_layer_bf16_delta(a, MB, NW, stream, shape) : launch_layer_bf16_first(a, MB, NW, stream, shape);
  }
  return delta ? launch_layer_f32_delta(a, MB, NW, stream, shape) : launch_layer_f32_first(a, MB, NW, stream, shape);
}

}  // namespace zeno
