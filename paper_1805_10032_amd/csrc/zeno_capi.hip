// C ABI of the Zeno library: argument checks, workspace layout and launch
// sequencing.  Every step of the path runs in the HIP kernels of this library;
// the host only validates and enqueues.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "zeno_internal.h"

// Scratch of zeno_score_static: a file-scope device array, one copy per GPU at that GPU's own
// address, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress, never an address to pass to a kernel.
static __device__ __align__(256) unsigned char scratch[ZENO_STATIC_SCRATCH_BYTES];

namespace {

using namespace zeno;

constexpr int kMaxPassRows = 128;  // samples per pass over G (four 32-row accumulator blocks)
constexpr int kMaxTileRows = 256;  // output features of the widest workgroup (eight waves x 32)

inline int pad64(int v) { return (v + 63) / 64 * 64; }
inline int blocks_for(int rows) { return rows <= 32 ? 1 : (rows <= 64 ? 2 : 4); }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Rows of the operand-order copy of a weight matrix.  The pass at x writes the copy one
// 32-row wave tile at a time for EVERY wave of its workgroups, also for waves whose rows lie
// beyond the layer (they store zeros), and the candidates' workgroups read it the same way;
// the widest workgroup of any launch covers kMaxTileRows features.
inline int wt_rows_alloc(int N, bool last) {
  const int cover = last ? N : pad64(N);
  return (cover + kMaxTileRows - 1) / kMaxTileRows * kMaxTileRows;
}

// Upper bound on the partial-norm slots per candidate of a layer N wide: its 32-row tiles, times up to 8 K
// slices while the launch's tiles x candidates x slices stay within the bytes of the partial-accumulator buffer.
inline int norm_slots_bound(int N, int m, int MB) {
  const int tiles = (pad64(N) + 31) / 32;
  const long long wgs = (long long)(kSlicePartialBytes / ((size_t)MB * 16 * 64 * sizeof(float)));
  long long sliced = wgs / (m > 0 ? m : 1);
  if (sliced > 8LL * tiles) sliced = 8LL * tiles;
  return tiles > sliced ? tiles : (int)sliced;
}

// Workspace layout, shared by the size query and the call itself.
struct Plan {
  int L, pass_rows, MB, n_pad, esize, P;
  size_t off_feat, off_hbase[ZENO_MAX_LAYERS], off_z0[ZENO_MAX_LAYERS];
  size_t off_wt[ZENO_MAX_LAYERS];  // W_l in operand order, layers after the first
  int wt_rows[ZENO_MAX_LAYERS];    // rows of that copy (features, rounded up to whole workgroup tiles)
  size_t off_dc[2], cand_stride, off_dz, off_norm, off_diff, total;
  size_t sz_hbase[ZENO_MAX_LAYERS], sz_z0[ZENO_MAX_LAYERS], sz_wt[ZENO_MAX_LAYERS], sz_dz;  // bytes of the slots
  // launches with K split over workgroups: partial accumulators and the arrival counters of the feature
  // tiles, shared by all launches of a pass (they run one after the other and leave the counters at zero)
  size_t off_slice_part, sz_slice_part, off_slice_cnt;
  int n_counters;
};

Plan make_plan(const zeno_model* mdl, int m, int n_r) {
  Plan p;
  std::memset(&p, 0, sizeof(p));
  const zeno_model_desc_t& D = mdl->desc;
  p.L = D.n_layers;
  p.pass_rows = n_r < kMaxPassRows ? n_r : kMaxPassRows;
  p.MB = blocks_for(p.pass_rows);
  p.n_pad = 32 * p.MB;
  p.esize = D.fwd == ZENO_FWD_BF16 ? 2 : 4;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  p.off_feat = take((size_t)p.n_pad * pad64(D.dims[0]) * p.esize);
  int max_np = 64;
  for (int l = 0; l < p.L; ++l) {
    const int N = D.dims[l + 1];
    p.sz_z0[l] = (size_t)p.pass_rows * N * sizeof(float);
    p.off_z0[l] = take(p.sz_z0[l]);
    if (l + 1 < p.L) {
      p.sz_hbase[l] = (size_t)p.n_pad * pad64(N) * p.esize;
      p.off_hbase[l] = take(p.sz_hbase[l]);
      if (pad64(N) > max_np) max_np = pad64(N);
    }
    if (l > 0) {
      // rows: whole feature tiles of the widest workgroup (256 features) that may carry the pass at x
      p.wt_rows[l] = wt_rows_alloc(N, l + 1 == p.L);
      p.sz_wt[l] = (size_t)p.wt_rows[l] * pad64(D.dims[l]) * p.esize;
      p.off_wt[l] = take(p.sz_wt[l]);
    }
    // upper bound on the partial-norm slots of this layer: the whole tiles of a launch, and a second range for the
    // (tile, slice) pairs of a sliced tail (at most 8 slices per 256-feature tile, i.e. one per 32 features)
    p.P += norm_slots_bound(N, m, p.MB) + norm_slots_bound(N, 1, p.MB);
  }
  p.n_counters = kMaxSliceGroups;
  p.sz_slice_part = kSlicePartialBytes;
  // a layer wide enough for eight-wave workgroups may run the tiles of its last candidates in K slices
  for (int l = 0; l < p.L; ++l) {
    const int cover = l + 1 == p.L ? D.dims[l + 1] : pad64(D.dims[l + 1]);
    if ((long long)((cover + kMaxTileRows - 1) / kMaxTileRows) * m >= 256 && tail_partial_bytes(p.MB) > p.sz_slice_part)
      p.sz_slice_part = tail_partial_bytes(p.MB);
  }
  p.off_slice_part = take(p.sz_slice_part);
  p.off_slice_cnt = take((size_t)p.n_counters * sizeof(unsigned int));
  p.cand_stride = align_up((size_t)p.n_pad * max_np * p.esize, 256);
  if (p.L > 1) {
    for (int i = 0; i < 2; ++i) p.off_dc[i] = take(p.cand_stride * m);
  }
  p.sz_dz = (size_t)m * p.pass_rows * D.dims[p.L] * sizeof(float);
  p.off_dz = take(p.sz_dz);
  p.off_norm = take((size_t)m * p.P * sizeof(double));
  p.off_diff = take((size_t)m * n_r * sizeof(double));
  p.total = off;
  return p;
}

#define ZENO_TRY(expr)                                \
  do {                                                \
    if ((expr) != hipSuccess) return ZENO_ERR_DEVICE; \
  } while (0)

// ---- optional per-launch timing (zeno_profile_enable / zeno_profile_collect):
// while enabled every kernel launch is bracketed by two HIP events recorded on
// the launch's own stream.
struct ProfEntry {
  hipEvent_t start, stop;
  zeno_profile_record_t rec;
};
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<ProfEntry> g_prof;

struct ProfScope {
  hipStream_t stream;
  int slot = -1;
  ProfScope(int kernel, int layer, double bytes, hipStream_t s) : stream(s) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof_on) return;
    ProfEntry e;
    if (hipEventCreate(&e.start) != hipSuccess) return;
    if (hipEventCreate(&e.stop) != hipSuccess) {
      (void)hipEventDestroy(e.start);
      return;
    }
    e.rec.kernel = kernel;
    e.rec.layer = layer;
    e.rec.ms = 0.f;
    e.rec.algorithmic_bytes = bytes;
    e.rec.waves = e.rec.k_split = e.rec.streaming = e.rec.row_blocks = e.rec.merged = e.rec.second = e.rec.k_slices = 0;
    e.rec.candidates = e.rec.tail_candidates = 0;
    (void)hipEventRecord(e.start, stream);
    g_prof.push_back(e);
    slot = (int)g_prof.size() - 1;
  }
  void set_shape(const LaunchShape& s, bool merged, bool second, int candidates, int tail) {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (slot >= (int)g_prof.size()) return;
    zeno_profile_record_t& r = g_prof[slot].rec;
    r.waves = s.waves;
    r.k_split = s.k_split;
    r.streaming = s.streaming;
    r.row_blocks = s.row_blocks;
    r.merged = merged ? 1 : 0;
    r.second = second ? 1 : 0;
    r.k_slices = s.k_slices;
    r.candidates = candidates;
    r.tail_candidates = tail;
  }
  ~ProfScope() {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (slot < (int)g_prof.size()) (void)hipEventRecord(g_prof[slot].stop, stream);
  }
};

zeno_status_t check_score_args(const zeno_model_t* model, const float* x, const float* G, int64_t ldg, int32_t m,
                               const zeno_batch_t* batch, float gamma, float rho, const float* scores) {
  if (model == nullptr || x == nullptr || G == nullptr || batch == nullptr || scores == nullptr)
    return ZENO_ERR_INVALID_ARG;
  if (m < 1 || m > ZENO_MAX_CANDIDATES || batch->n_r < 1 || ldg < model->d) return ZENO_ERR_INVALID_ARG;
  if (!std::isfinite(gamma) || gamma < 0.f || !std::isfinite(rho) || rho < 0.f) return ZENO_ERR_INVALID_ARG;
  const zeno_model_desc_t& D = model->desc;
  if (batch->features == nullptr) return ZENO_ERR_INVALID_ARG;
  if (D.loss == ZENO_LOSS_SOFTMAX_CE && batch->labels == nullptr) return ZENO_ERR_INVALID_ARG;
  if (D.loss == ZENO_LOSS_SQUARED && batch->targets == nullptr) return ZENO_ERR_INVALID_ARG;
  if (!aligned(x, 4) || !aligned(G, 4) || !aligned(scores, 4) || !aligned(batch->features, 4) ||
      !aligned(batch->labels, 4) || !aligned(batch->targets, 4))
    return ZENO_ERR_INVALID_ARG;
  return ZENO_OK;
}

// One launch of the layer kernel as the sequence plans it.
struct Launch {
  LayerArgs a;
  bool delta;     // candidates carry the second product
  int kernel;     // zeno_kernel_t, for the per-launch timing
  int layer;
  double bytes;   // algorithmic bytes
  int wt_layer;   // layer whose operand-order copy of W the launch writes, or -1
  int base_layer; // layer the pass at x runs through in this launch, or -1
};

// The layer launches of one pass over G (rows samples): [pass at x, layer 0], then for
// every layer l the candidates' layer l, with the pass at x through layer l+1 (whose
// input the previous launch completed) either inside that launch or as a launch of its
// own in front of it.  A single-layer model needs one launch.  *P_out receives the
// partial-norm slots per candidate.  query_device = false plans without asking the
// device for occupancies (every merge is then planned as merged, the wider case).
std::vector<Launch> layer_sequence(const zeno_model* model, const Plan& p, const float* x, const float* G, int64_t ldg,
                                   int m, float gamma, unsigned char* ws, int rows, bool first_pass, int* P_out,
                                   bool query_device = true) {
  const zeno_model_desc_t& D = model->desc;
  const bool bf16 = D.fwd == ZENO_FWD_BF16;
  const int L = p.L;
  auto make_job = [&](int l) {
    LayerJob j;
    std::memset(&j, 0, sizeof(j));
    j.w_off = model->w_off[l];
    j.b_off = model->b_off[l];
    j.N = D.dims[l + 1];
    j.K = D.dims[l];
    j.Kp = pad64(j.K);
    j.Np = pad64(j.N);
    j.last = (l + 1 == L);
    j.A_base = l == 0 ? ws + p.off_feat : ws + p.off_hbase[l - 1];
    j.Wt = l > 0 ? ws + p.off_wt[l] : nullptr;
    j.Z0 = reinterpret_cast<float*>(ws + p.off_z0[l]);
    j.H_base = j.last ? nullptr : ws + p.off_hbase[l];
    return j;
  };
  // bytes of layer l's block in one parameter vector (what one source streams)
  auto layer_bytes = [&](int l) {
    return 4.0 * ((double)D.dims[l + 1] * D.dims[l] + (model->b_off[l] >= 0 ? D.dims[l + 1] : 0));
  };
  LayerArgs common;
  std::memset(&common, 0, sizeof(common));
  common.G = G;
  common.x = x;
  common.ldg = ldg;
  common.dZ = reinterpret_cast<float*>(ws + p.off_dz);
  common.gamma = gamma;
  common.neg_inv_gamma = gamma > 0.f ? -1.0f / gamma : 0.f;
  common.n_r = rows;
  common.slice_partials = reinterpret_cast<float*>(ws + p.off_slice_part);
  common.slice_counters = reinterpret_cast<unsigned int*>(ws + p.off_slice_cnt);

  std::vector<Launch> seq;
  if (L > 1) {
    Launch b;
    b.a = common;
    b.a.has_base = 1;
    b.a.bj = make_job(0);
    b.delta = false;
    b.kernel = ZENO_KERNEL_LAYER_BASE;
    b.layer = 0;
    b.bytes = layer_bytes(0);
    b.wt_layer = -1;
    b.base_layer = 0;
    seq.push_back(b);
  }
  for (int l = 0; l < L; ++l) {
    Launch c;
    c.a = common;
    c.a.n_cand = m;
    c.a.cj = make_job(l);
    c.a.norm_partials = first_pass ? reinterpret_cast<double*>(ws + p.off_norm) : nullptr;
    c.delta = l > 0;
    c.kernel = ZENO_KERNEL_LAYER_CAND;
    c.layer = l;
    c.bytes = layer_bytes(l) * m;
    c.wt_layer = -1;
    c.base_layer = -1;
    if (L == 1) {
      c.a.has_base = 1;
      c.a.bj = make_job(0);
      c.base_layer = 0;
      c.bytes += layer_bytes(0);
      seq.push_back(c);
      continue;
    }
    c.a.D_cand = l == 0 ? nullptr : ws + p.off_dc[(l - 1) & 1];
    c.a.A_stride = (long long)p.cand_stride;
    c.a.Dl_cand = ws + p.off_dc[l & 1];
    c.a.H_stride = (long long)p.cand_stride;
    if (l + 1 < L) {
      c.a.has_base = 1;
      c.a.bj = make_job(l + 1);
    }
    // A launch whose last round of eight-wave workgroups would be partly empty runs the tiles of that round's
    // candidates, and the pass at x, in K slices at its end.
    int tail_main = m;
    const int tail_slices = query_device ? layer_tail_slices(c.a, bf16, l > 0, p.MB, &tail_main) : 0;
    if (tail_slices >= 2) {
      c.a.tail_cand = m - tail_main;
      c.a.tail_slices = tail_slices;
      if (l + 1 < L) {
        c.bytes += layer_bytes(l + 1);
        c.wt_layer = l + 1;
        c.base_layer = l + 1;
      }
      seq.push_back(c);
      continue;
    }
    if (l + 1 < L) {
      if (!query_device || layer_merge_pays(c.a, bf16, l > 0, p.MB)) {
        c.bytes += layer_bytes(l + 1);
        c.wt_layer = l + 1;
        c.base_layer = l + 1;
      } else {
        // the extra workgroups would cost a whole extra round: run the pass at x on its own first
        Launch b;
        b.a = common;
        b.a.has_base = 1;
        b.a.bj = c.a.bj;
        b.delta = false;
        b.kernel = ZENO_KERNEL_LAYER_BASE;
        b.layer = l + 1;
        b.bytes = layer_bytes(l + 1);
        b.wt_layer = l + 1;
        b.base_layer = l + 1;
        seq.push_back(b);
        c.a.has_base = 0;
      }
    }
    seq.push_back(c);
  }
  // Partial-norm slots of the candidate launches, now that it is known which of them also carry the pass at x
  // (that changes how a launch of one-wave tiles splits K): a launch gets feature tiles x K slices slots.
  int P = 0;
  for (Launch& c : seq) {
    if (c.a.n_cand <= 0) continue;
    c.a.p_off = P;
    if (c.a.tail_slices >= 2) c.a.tail_p_off = P + (pad64(D.dims[c.layer + 1]) + kMaxTileRows - 1) / kMaxTileRows;
    P += query_device ? layer_tiles(c.a, bf16, c.delta, p.MB) : norm_slots_bound(D.dims[c.layer + 1], m, p.MB);
  }
  for (Launch& c : seq)
    if (c.a.n_cand > 0) c.a.P = P;
  *P_out = P;
  return seq;
}

// Does everything a launch writes with NW waves per workgroup lie inside its workspace slot?
bool launch_fits(const Plan& p, const Launch& L, int NW, bool device) {
  const bool bf16 = p.esize == 2;
  const LayerExtents e = layer_extents(L.a, bf16, L.delta, p.MB, NW, device);
  if (L.wt_layer >= 0 ? (size_t)e.wt_bytes > p.sz_wt[L.wt_layer] : e.wt_bytes != 0) return false;
  if (L.base_layer >= 0) {
    if ((size_t)e.z0_floats * sizeof(float) > p.sz_z0[L.base_layer]) return false;
    if (L.base_layer + 1 < p.L && (size_t)e.hbase_bytes > p.sz_hbase[L.base_layer]) return false;
  }
  if (L.a.n_cand > 0) {
    if ((size_t)e.d_bytes_per_cand > p.cand_stride) return false;
    if ((size_t)e.dz_floats * sizeof(float) > p.sz_dz) return false;
    if (L.a.P > p.P || L.a.p_off + e.norm_slots > L.a.P) return false;
  }
  if ((size_t)e.slice_bytes > p.sz_slice_part || e.slice_counters > p.n_counters) return false;
  return true;
}

zeno_status_t score_enqueue(const zeno_model* model, const Plan& p, const float* x, const float* G, int64_t ldg, int m,
                            const zeno_batch_t* batch, float gamma, float rho, float* scores, unsigned char* ws,
                            hipStream_t stream) {
  const zeno_model_desc_t& D = model->desc;
  const bool bf16 = D.fwd == ZENO_FWD_BF16;
  const int L = p.L, n_r = batch->n_r, C = D.dims[L];
  double* norm_partials = reinterpret_cast<double*>(ws + p.off_norm);
  double* sample_diff = reinterpret_cast<double*>(ws + p.off_diff);
  float* dZ = reinterpret_cast<float*>(ws + p.off_dz);
  int P = 0;
  for (int begin = 0; begin < n_r; begin += p.pass_rows) {
    const int rows = (n_r - begin) < p.pass_rows ? (n_r - begin) : p.pass_rows;
    const std::vector<Launch> seq = layer_sequence(model, p, x, G, ldg, m, gamma, ws, rows, begin == 0, &P);
    // nothing is enqueued for a pass unless every launch of it stays inside its slots
    for (const Launch& l : seq)
      if (!launch_fits(p, l, layer_nw(l.a, bf16, l.delta, p.MB), true)) return ZENO_ERR_WORKSPACE;
    {
      ProfScope ps(ZENO_KERNEL_PACK, 0, 4.0 * rows * D.dims[0], stream);
      ZENO_TRY(launch_pack_features(batch->features + (size_t)begin * D.dims[0], rows, D.dims[0], pad64(D.dims[0]),
                                    p.MB, bf16, ws + p.off_feat,
                                    reinterpret_cast<unsigned int*>(ws + p.off_slice_cnt), p.n_counters,
                                    begin == 0 ? norm_partials : nullptr, begin == 0 ? (long long)m * P : 0, stream));
    }
    for (const Launch& l : seq) {
      ProfScope ps(l.kernel, l.layer, l.bytes, stream);
      LaunchShape shape;
      ZENO_TRY(launch_layer(l.a, bf16, l.delta, p.MB, stream, &shape));
      ps.set_shape(shape, l.a.n_cand > 0 && l.a.has_base, l.a.n_cand > 0 && l.delta, l.a.n_cand, l.a.tail_cand);
    }
    ProfScope ps(ZENO_KERNEL_LOSS, 0, 4.0 * (m + 1) * rows * C, stream);
    ZENO_TRY(launch_loss(reinterpret_cast<const float*>(ws + p.off_z0[L - 1]), dZ, batch->labels, batch->targets,
                         D.loss, m, n_r, begin, rows, C, sample_diff, stream));
  }
  ProfScope ps(ZENO_KERNEL_COMBINE, 0, 8.0 * m * (n_r + P), stream);
  ZENO_TRY(launch_score_combine(sample_diff, norm_partials, P, m, n_r, rho, scores, stream));
  return ZENO_OK;
}


// ---- convolutional models: workspace layout and launch sequence
constexpr int kConvNormBlocks = 8;   // pieces the squared norm of a candidate's convolution kernels is summed in

struct CnnPlan {
  int n_conv, MB, n_pad, Kfc, Kp, P;
  size_t off_z0[ZENO_MAX_CONV], off_h0[ZENO_MAX_CONV], off_d[2], d_stride;  // maps (floats per candidate in d_stride)
  size_t off_h0t, off_dt, dt_stride, sz_h0t;                                  // operands of the fully connected layer
  size_t off_wt, off_z0fc, off_dz, off_norm, off_diff, total;
  size_t off_slice_part, off_slice_cnt, sz_slice_cnt;   // K slices of the fully connected layer's launches
};

CnnPlan make_cnn_plan(const zeno_model* mdl, int m, int n_r) {
  CnnPlan p;
  std::memset(&p, 0, sizeof(p));
  const int C = mdl->cnn.n_conv;
  p.n_conv = C;
  p.MB = blocks_for(n_r);
  p.n_pad = 32 * p.MB;
  p.Kfc = mdl->map_h[C] * mdl->map_w[C] * mdl->map_c[C];
  p.Kp = pad64(p.Kfc);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  size_t max_map = 0;
  for (int l = 0; l < C; ++l) {
    const size_t map = (size_t)n_r * mdl->map_h[l + 1] * mdl->map_w[l + 1] * mdl->map_c[l + 1];
    p.off_z0[l] = take(map * sizeof(float));
    if (l + 1 < C) {
      p.off_h0[l] = take(map * sizeof(float));
      if (map > max_map) max_map = map;
    }
  }
  p.d_stride = align_up(max_map * sizeof(float), 256) / sizeof(float);
  if (C > 1)
    for (int i = 0; i < 2; ++i) p.off_d[i] = take(p.d_stride * sizeof(float) * m);
  p.sz_h0t = (size_t)p.n_pad * p.Kp * sizeof(float);
  p.off_h0t = take(p.sz_h0t);
  p.dt_stride = align_up(p.sz_h0t, 256);
  p.off_dt = take(p.dt_stride * m);
  const int N = mdl->cnn.fc_out;
  p.off_wt = take((size_t)wt_rows_alloc(N, true) * p.Kp * sizeof(float));
  p.off_z0fc = take((size_t)n_r * N * sizeof(float));
  p.off_dz = take((size_t)m * n_r * N * sizeof(float));
  p.P = norm_slots_bound(N, m, p.MB) + kConvNormBlocks;
  p.off_norm = take((size_t)m * p.P * sizeof(double));
  p.off_slice_part = take(kSlicePartialBytes);
  p.sz_slice_cnt = align_up((size_t)kMaxSliceGroups * sizeof(unsigned int), 256);
  p.off_slice_cnt = take(p.sz_slice_cnt);
  p.off_diff = take((size_t)m * n_r * sizeof(double));
  p.total = off;
  return p;
}

zeno_status_t cnn_score_enqueue(const zeno_model* mdl, const CnnPlan& p, const float* x, const float* G, int64_t ldg,
                                int m, const zeno_batch_t* batch, float gamma, float rho, float* scores,
                                unsigned char* ws, hipStream_t stream) {
  const int C = p.n_conv, n_r = batch->n_r, N = mdl->cnn.fc_out;
  const float neg_inv_gamma = gamma > 0.f ? -1.0f / gamma : 0.f;
  double* norm_partials = reinterpret_cast<double*>(ws + p.off_norm);
  double* sample_diff = reinterpret_cast<double*>(ws + p.off_diff);
  float* dZ = reinterpret_cast<float*>(ws + p.off_dz);

  // the padded columns of the fully connected layer's operands (beyond K) must hold zeros, not whatever the
  // workspace held (they meet the zeros of the masked weight tile, and 0 x NaN is NaN); the convolutions only
  // write the live entries
  // (rows beyond n_r may hold anything: a sample's row only reaches its own, discarded, results)
  {
    ProfScope ps(ZENO_KERNEL_AUX, 2, 0.0, stream);
    ZENO_TRY(launch_fill_zero(ws + p.off_slice_cnt, p.sz_slice_cnt, stream));   // arrival counters start at zero
  }
  if (p.Kp != p.Kfc) {
    ProfScope ps(ZENO_KERNEL_AUX, 0, 0.0, stream);
    ZENO_TRY(launch_fill_zero(ws + p.off_h0t, p.sz_h0t, stream));
    ZENO_TRY(launch_fill_zero(ws + p.off_dt, p.dt_stride * m, stream));
  }
  auto conv_args = [&](int l) {
    ConvArgs a;
    std::memset(&a, 0, sizeof(a));
    a.G = G;
    a.x = x;
    a.ldg = ldg;
    a.n_r = n_r;
    a.L.w_off = mdl->conv_w_off[l];
    a.L.b_off = mdl->conv_b_off[l];
    a.L.Hin = mdl->map_h[l];
    a.L.Win = mdl->map_w[l];
    a.L.Cin = mdl->map_c[l];
    a.L.Hout = mdl->map_h[l + 1];
    a.L.Wout = mdl->map_w[l + 1];
    a.L.Cout = mdl->map_c[l + 1];
    a.L.stride = mdl->cnn.conv_stride[l];
    a.H0_in = l == 0 ? batch->features : reinterpret_cast<const float*>(ws + p.off_h0[l - 1]);
    a.Z0 = reinterpret_cast<float*>(ws + p.off_z0[l]);
    a.tiled_out = l + 1 == C;
    a.Kp_fc = p.Kp;
    a.gamma = gamma;
    a.neg_inv_gamma = neg_inv_gamma;
    return a;
  };
  auto conv_flops = [&](int l) {   // reported in place of bytes: 2 * positions * 9 c_in * c_out per source
    return 2.0 * n_r * mdl->map_h[l + 1] * mdl->map_w[l + 1] * 9.0 * mdl->map_c[l] * mdl->map_c[l + 1];
  };
  // pass at x through the convolutions, then the candidates (layer l of the candidates needs Z0 of layer l
  // and the input map of layer l, both written by the pass at x)
  for (int l = 0; l < C; ++l) {
    ConvArgs a = conv_args(l);
    a.out = l + 1 == C ? reinterpret_cast<float*>(ws + p.off_h0t) : reinterpret_cast<float*>(ws + p.off_h0[l]);
    ProfScope ps(ZENO_KERNEL_CONV_BASE, l, conv_flops(l), stream);
    ZENO_TRY(launch_conv(a, stream));
  }
  for (int l = 0; l < C; ++l) {
    ConvArgs a = conv_args(l);
    a.n_cand = m;
    if (l > 0) {
      a.D_in = reinterpret_cast<const float*>(ws + p.off_d[(l - 1) & 1]);
      a.D_in_stride = (long long)p.d_stride;
    }
    if (l + 1 == C) {
      a.out = reinterpret_cast<float*>(ws + p.off_dt);
      a.out_stride = (long long)(p.dt_stride / sizeof(float));
    } else {
      a.out = reinterpret_cast<float*>(ws + p.off_d[l & 1]);
      a.out_stride = (long long)p.d_stride;
    }
    ProfScope ps(ZENO_KERNEL_CONV_CAND, l, conv_flops(l) * m * (l > 0 ? 2 : 1), stream);
    ZENO_TRY(launch_conv(a, stream));
  }
  // the fully connected layer on the streaming layer kernel (fp32, with the second product)
  LayerJob j;
  std::memset(&j, 0, sizeof(j));
  j.w_off = mdl->w_off[0];
  j.b_off = mdl->b_off[0];
  j.N = N;
  j.K = p.Kfc;
  j.Kp = p.Kp;
  j.Np = pad64(N);
  j.last = 1;
  j.A_base = ws + p.off_h0t;
  j.Wt = ws + p.off_wt;
  j.Z0 = reinterpret_cast<float*>(ws + p.off_z0fc);
  LayerArgs common;
  std::memset(&common, 0, sizeof(common));
  common.G = G;
  common.x = x;
  common.ldg = ldg;
  common.dZ = dZ;
  common.gamma = gamma;
  common.neg_inv_gamma = neg_inv_gamma;
  common.n_r = n_r;
  common.slice_partials = reinterpret_cast<float*>(ws + p.off_slice_part);
  common.slice_counters = reinterpret_cast<unsigned int*>(ws + p.off_slice_cnt);
  const double fc_bytes = 4.0 * ((double)N * p.Kfc + (j.b_off >= 0 ? N : 0));
  {
    LayerArgs b = common;
    b.has_base = 1;
    b.bj = j;
    ProfScope ps(ZENO_KERNEL_LAYER_BASE, C, fc_bytes, stream);
    ZENO_TRY(launch_layer(b, false, false, p.MB, stream));
  }
  LayerArgs c = common;
  c.n_cand = m;
  c.cj = j;
  c.D_cand = ws + p.off_dt;
  c.A_stride = (long long)p.dt_stride;
  c.norm_partials = norm_partials;
  c.P = p.P;
  c.p_off = 0;
  const int fc_tiles = layer_tiles(c, false, true, p.MB);
  if (fc_tiles + kConvNormBlocks > p.P) return ZENO_ERR_WORKSPACE;
  {
    ProfScope ps(ZENO_KERNEL_LAYER_CAND, C, fc_bytes * m, stream);
    ZENO_TRY(launch_layer(c, false, true, p.MB, stream));
  }
  // ||u||^2 runs over all d coordinates: the fully connected block was summed by the layer kernel, the
  // convolutions' kernels and biases (the first mdl->w_off[0] coordinates) are summed here; slots that no
  // launch writes are cleared
  {
    ProfScope ps(ZENO_KERNEL_AUX, 1, 4.0 * (double)mdl->w_off[0] * m, stream);
    ZENO_TRY(launch_sumsq(G, ldg, m, 0, mdl->w_off[0], kConvNormBlocks, norm_partials, p.P, fc_tiles, stream));
  }
  const int P_used = fc_tiles + kConvNormBlocks;
  {
    ProfScope ps(ZENO_KERNEL_LOSS, 0, 4.0 * (m + 1) * n_r * N, stream);
    ZENO_TRY(launch_loss(j.Z0, dZ, batch->labels, batch->targets, mdl->cnn.loss, m, n_r, 0, n_r, N, sample_diff, stream));
  }
  ProfScope ps(ZENO_KERNEL_COMBINE, 0, 8.0 * m * (n_r + P_used), stream);
  ZENO_TRY(launch_score_combine_strided(sample_diff, norm_partials, p.P, P_used, m, n_r, rho, scores, stream));
  return ZENO_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch(unsigned char** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = reinterpret_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

zeno_status_t zeno_profile_enable(int32_t enable) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof_on = enable != 0;
  return ZENO_OK;
}

int32_t zeno_profile_collect(zeno_profile_record_t* records, int32_t max_records) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  int32_t n = 0;
  for (ProfEntry& e : g_prof) {
    float ms = 0.f;
    if (hipEventSynchronize(e.stop) == hipSuccess && hipEventElapsedTime(&ms, e.start, e.stop) == hipSuccess) {
      e.rec.ms = ms;
      if (records != nullptr && n < max_records) records[n++] = e.rec;
    }
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  g_prof.clear();
  return n;
}

zeno_status_t zeno_model_create(const zeno_model_desc_t* desc, zeno_model_t** out) {
  if (desc == nullptr || out == nullptr) return ZENO_ERR_INVALID_ARG;
  if (desc->n_layers < 1 || desc->n_layers > ZENO_MAX_LAYERS) return ZENO_ERR_INVALID_ARG;
  for (int l = 0; l <= desc->n_layers; ++l)
    if (desc->dims[l] < 1) return ZENO_ERR_INVALID_ARG;
  if (desc->has_bias != 0 && desc->has_bias != 1) return ZENO_ERR_INVALID_ARG;
  if (desc->loss != ZENO_LOSS_SQUARED && desc->loss != ZENO_LOSS_SOFTMAX_CE) return ZENO_ERR_INVALID_ARG;
  if (desc->fwd != ZENO_FWD_FP32 && desc->fwd != ZENO_FWD_BF16) return ZENO_ERR_INVALID_ARG;
  if (desc->loss == ZENO_LOSS_SQUARED && desc->dims[desc->n_layers] != 1) return ZENO_ERR_INVALID_ARG;
  zeno_model* mdl = new (std::nothrow) zeno_model;
  if (mdl == nullptr) return ZENO_ERR_HOST_MEMORY;
  std::memset(mdl, 0, sizeof(*mdl));
  mdl->kind = 0;
  mdl->desc = *desc;
  int64_t off = 0;
  for (int l = 0; l < desc->n_layers; ++l) {
    mdl->w_off[l] = off;
    off += (int64_t)desc->dims[l + 1] * desc->dims[l];
    mdl->b_off[l] = -1;
    if (desc->has_bias) {
      mdl->b_off[l] = off;
      off += desc->dims[l + 1];
    }
  }
  mdl->d = off;
  *out = mdl;
  return ZENO_OK;
}

zeno_status_t zeno_cnn_model_create(const zeno_cnn_desc_t* desc, zeno_model_t** out) {
  if (desc == nullptr || out == nullptr) return ZENO_ERR_INVALID_ARG;
  if (desc->n_conv < 1 || desc->n_conv > ZENO_MAX_CONV) return ZENO_ERR_INVALID_ARG;
  if (desc->in_h < 1 || desc->in_w < 1 || desc->in_c < 1 || desc->fc_out < 1) return ZENO_ERR_INVALID_ARG;
  if (desc->has_bias != 0 && desc->has_bias != 1) return ZENO_ERR_INVALID_ARG;
  if (desc->loss != ZENO_LOSS_SQUARED && desc->loss != ZENO_LOSS_SOFTMAX_CE) return ZENO_ERR_INVALID_ARG;
  if (desc->loss == ZENO_LOSS_SQUARED && desc->fc_out != 1) return ZENO_ERR_INVALID_ARG;
  for (int l = 0; l < desc->n_conv; ++l)
    if (desc->conv_c[l] < 1 || (desc->conv_stride[l] != 1 && desc->conv_stride[l] != 2)) return ZENO_ERR_INVALID_ARG;
  zeno_model* mdl = new (std::nothrow) zeno_model;
  if (mdl == nullptr) return ZENO_ERR_HOST_MEMORY;
  std::memset(mdl, 0, sizeof(*mdl));
  mdl->kind = 1;
  mdl->cnn = *desc;
  mdl->map_h[0] = desc->in_h;
  mdl->map_w[0] = desc->in_w;
  mdl->map_c[0] = desc->in_c;
  int64_t off = 0;
  for (int l = 0; l < desc->n_conv; ++l) {
    mdl->map_h[l + 1] = (mdl->map_h[l] - 1) / desc->conv_stride[l] + 1;
    mdl->map_w[l + 1] = (mdl->map_w[l] - 1) / desc->conv_stride[l] + 1;
    mdl->map_c[l + 1] = desc->conv_c[l];
    mdl->conv_w_off[l] = off;
    off += (int64_t)desc->conv_c[l] * 9 * mdl->map_c[l];
    mdl->conv_b_off[l] = -1;
    if (desc->has_bias) {
      mdl->conv_b_off[l] = off;
      off += desc->conv_c[l];
    }
  }
  const int C = desc->n_conv;
  const int64_t kfc = (int64_t)mdl->map_h[C] * mdl->map_w[C] * mdl->map_c[C];
  if (kfc > (int64_t)1 << 30) {
    delete mdl;
    return ZENO_ERR_INVALID_ARG;
  }
  // the fully connected layer, described as a one-layer chain for the code that sizes things by `desc`
  mdl->desc.n_layers = 1;
  mdl->desc.dims[0] = (int32_t)kfc;
  mdl->desc.dims[1] = desc->fc_out;
  mdl->desc.has_bias = desc->has_bias;
  mdl->desc.loss = desc->loss;
  mdl->desc.fwd = ZENO_FWD_FP32;
  mdl->w_off[0] = off;
  off += kfc * desc->fc_out;
  mdl->b_off[0] = -1;
  if (desc->has_bias) {
    mdl->b_off[0] = off;
    off += desc->fc_out;
  }
  mdl->d = off;
  *out = mdl;
  return ZENO_OK;
}

void zeno_model_destroy(zeno_model_t* model) { delete model; }

int64_t zeno_model_num_params(const zeno_model_t* model) { return model == nullptr ? 0 : model->d; }

size_t zeno_score_workspace_bytes(const zeno_model_t* model, int32_t m, int32_t n_r) {
  if (model == nullptr || m < 1 || m > ZENO_MAX_CANDIDATES || n_r < 1) return 0;
  if (model->kind == 1) return n_r > kMaxPassRows ? 0 : make_cnn_plan(model, m, n_r).total;
  return make_plan(model, m, n_r).total;
}

zeno_status_t zeno_score(const zeno_model_t* model, const float* x, const float* G, int64_t ldg, int32_t m,
                         const zeno_batch_t* batch, float gamma, float rho, float* scores, void* workspace,
                         size_t workspace_bytes, void* stream_) {
  zeno_status_t st = check_score_args(model, x, G, ldg, m, batch, gamma, rho, scores);
  if (st != ZENO_OK) return st;
  if (model->kind == 1) {
    if (batch->n_r > kMaxPassRows) return ZENO_ERR_UNSUPPORTED;
    const CnnPlan cp = make_cnn_plan(model, m, batch->n_r);
    if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < cp.total) return ZENO_ERR_WORKSPACE;
    return cnn_score_enqueue(model, cp, x, G, ldg, m, batch, gamma, rho, scores, reinterpret_cast<unsigned char*>(workspace),
                             reinterpret_cast<hipStream_t>(stream_));
  }
  const Plan p = make_plan(model, m, batch->n_r);
  if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < p.total) return ZENO_ERR_WORKSPACE;
  return score_enqueue(model, p, x, G, ldg, m, batch, gamma, rho, scores, reinterpret_cast<unsigned char*>(workspace),
                       reinterpret_cast<hipStream_t>(stream_));
}

zeno_status_t zeno_score_static(const zeno_model_t* model, const float* x, const float* G, int64_t ldg, int32_t m,
                                const zeno_batch_t* batch, float gamma, float rho, float* scores, void* stream_) {
  zeno_status_t st = check_score_args(model, x, G, ldg, m, batch, gamma, rho, scores);
  if (st != ZENO_OK) return st;
  if (model->kind == 1) {
    if (batch->n_r > kMaxPassRows) return ZENO_ERR_UNSUPPORTED;
    const CnnPlan cp = make_cnn_plan(model, m, batch->n_r);
    if (cp.total > (size_t)ZENO_STATIC_SCRATCH_BYTES) return ZENO_ERR_UNSUPPORTED;
    unsigned char* cws = nullptr;
    if (static_scratch(&cws) != hipSuccess) return ZENO_ERR_DEVICE;
    return cnn_score_enqueue(model, cp, x, G, ldg, m, batch, gamma, rho, scores, cws, reinterpret_cast<hipStream_t>(stream_));
  }
  const Plan p = make_plan(model, m, batch->n_r);
  if (p.total > (size_t)ZENO_STATIC_SCRATCH_BYTES) return ZENO_ERR_UNSUPPORTED;
  unsigned char* ws = nullptr;
  if (static_scratch(&ws) != hipSuccess) return ZENO_ERR_DEVICE;
  // Every slot of the layout is written by an earlier launch of the same call before a later one
  // reads it, so nothing left behind by the previous call has to be cleared.
  return score_enqueue(model, p, x, G, ldg, m, batch, gamma, rho, scores, ws, reinterpret_cast<hipStream_t>(stream_));
}

zeno_status_t zeno_score_plan_check(const zeno_model_t* model, int32_t m, int32_t n_r) {
  if (model == nullptr || m < 1 || m > ZENO_MAX_CANDIDATES || n_r < 1) return ZENO_ERR_INVALID_ARG;
  if (model->kind != 0) return ZENO_ERR_UNSUPPORTED;
  const Plan p = make_plan(model, m, n_r);
  // a fictitious, suitably aligned workspace address: nothing is dereferenced
  unsigned char* ws = reinterpret_cast<unsigned char*>(uintptr_t(1) << 40);
  const float* fake = reinterpret_cast<const float*>(uintptr_t(1) << 30);
  zeno_batch_t batch;
  std::memset(&batch, 0, sizeof(batch));
  batch.n_r = n_r;
  batch.features = fake;
  static const int widths[3] = {1, 4, 8};
  for (int begin = 0; begin < n_r; begin += p.pass_rows) {
    const int rows = (n_r - begin) < p.pass_rows ? (n_r - begin) : p.pass_rows;
    int P = 0;
    const std::vector<Launch> seq = layer_sequence(model, p, fake, fake, model->d, m, 0.1f, ws, rows, begin == 0, &P,
                                                   /*query_device=*/false);
    for (const Launch& L : seq)
      for (int NW : widths)
        if (!launch_fits(p, L, NW, false)) return ZENO_ERR_WORKSPACE;
  }
  return ZENO_OK;
}

zeno_status_t zeno_aggregate(const float* G, int64_t ldg, const float* scores, int32_t m, int64_t d, int32_t b,
                             float* out, int32_t* selected, void* stream) {
  if (G == nullptr || scores == nullptr || out == nullptr) return ZENO_ERR_INVALID_ARG;
  if (m < 1 || m > ZENO_MAX_CANDIDATES || b < 0 || b >= m || d < 1 || ldg < d) return ZENO_ERR_INVALID_ARG;
  if (!aligned(G, 4) || !aligned(scores, 4) || !aligned(out, 4) || !aligned(selected, 4)) return ZENO_ERR_INVALID_ARG;
  ProfScope ps(ZENO_KERNEL_AVERAGE, 0, 4.0 * (double)d * (m - b + 1), reinterpret_cast<hipStream_t>(stream));
  ZENO_TRY(launch_masked_average(G, ldg, scores, m, d, b, out, selected, reinterpret_cast<hipStream_t>(stream)));
  return ZENO_OK;
}

zeno_status_t zeno_aggregate_update(const float* G, int64_t ldg, const float* scores, int32_t m, int64_t d,
                                    int32_t b, float gamma, const float* x, float* x_next, float* out,
                                    int32_t* selected, void* stream) {
  if (G == nullptr || scores == nullptr || x == nullptr || x_next == nullptr) return ZENO_ERR_INVALID_ARG;
  if (m < 1 || m > ZENO_MAX_CANDIDATES || b < 0 || b >= m || d < 1 || ldg < d) return ZENO_ERR_INVALID_ARG;
  if (!std::isfinite(gamma) || gamma < 0.f) return ZENO_ERR_INVALID_ARG;
  if (!aligned(G, 4) || !aligned(scores, 4) || !aligned(x, 4) || !aligned(x_next, 4) || !aligned(out, 4) ||
      !aligned(selected, 4))
    return ZENO_ERR_INVALID_ARG;
  ProfScope ps(ZENO_KERNEL_AVERAGE_UPDATE, 0, 4.0 * (double)d * (m - b + 2 + (out != nullptr ? 1 : 0)),
               reinterpret_cast<hipStream_t>(stream));
  ZENO_TRY(launch_masked_average(G, ldg, scores, m, d, b, out, selected, reinterpret_cast<hipStream_t>(stream), gamma,
                                 x, x_next));
  return ZENO_OK;
}

zeno_status_t zeno_mean(const float* G, int64_t ldg, int32_t m, int64_t d, float* out, void* stream) {
  if (G == nullptr || out == nullptr) return ZENO_ERR_INVALID_ARG;
  if (m < 1 || m > ZENO_MAX_CANDIDATES || d < 1 || ldg < d) return ZENO_ERR_INVALID_ARG;
  if (!aligned(G, 4) || !aligned(out, 4)) return ZENO_ERR_INVALID_ARG;
  ProfScope ps(ZENO_KERNEL_MEAN, 0, 4.0 * (double)d * (m + 1), reinterpret_cast<hipStream_t>(stream));
  ZENO_TRY(launch_masked_average(G, ldg, nullptr, m, d, 0, out, nullptr, reinterpret_cast<hipStream_t>(stream)));
  return ZENO_OK;
}

zeno_status_t zeno_median(const float* G, int64_t ldg, int32_t m, int64_t d, float* out, void* stream) {
  if (G == nullptr || out == nullptr) return ZENO_ERR_INVALID_ARG;
  if (m < 1 || m > ZENO_MAX_CANDIDATES || d < 1 || ldg < d) return ZENO_ERR_INVALID_ARG;
  if (!aligned(G, 4) || !aligned(out, 4)) return ZENO_ERR_INVALID_ARG;
  ProfScope ps(ZENO_KERNEL_MEDIAN, 0, 4.0 * (double)d * (m + 1), reinterpret_cast<hipStream_t>(stream));
  if (m > 128) {
    // more rows than the sorting networks in registers hold: rank selection on keys kept in LDS
    ZENO_TRY(launch_median_select(G, ldg, m, d, out, reinterpret_cast<hipStream_t>(stream)));
    return ZENO_OK;
  }
  ZENO_TRY(launch_median(G, ldg, m, d, out, reinterpret_cast<hipStream_t>(stream)));
  return ZENO_OK;
}

size_t zeno_krum_workspace_bytes(int32_t m) {
  if (m < 3 || m > 128) return 0;
  return krum_workspace_bytes(m);
}

zeno_status_t zeno_krum(const float* G, int64_t ldg, int32_t m, int64_t d, int32_t b, float* out, int32_t* chosen,
                        float* krum_scores, void* workspace, size_t workspace_bytes, void* stream) {
  if (G == nullptr || out == nullptr || chosen == nullptr) return ZENO_ERR_INVALID_ARG;
  if (m < 3 || m > ZENO_MAX_CANDIDATES || b < 0 || m - b - 2 < 1 || d < 1 || ldg < d) return ZENO_ERR_INVALID_ARG;
  if (!aligned(G, 4) || !aligned(out, 4) || !aligned(chosen, 4) || !aligned(krum_scores, 4)) return ZENO_ERR_INVALID_ARG;
  if (m > 128) return ZENO_ERR_UNSUPPORTED;
  if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < krum_workspace_bytes(m))
    return ZENO_ERR_WORKSPACE;
  ProfScope ps(ZENO_KERNEL_KRUM, 0, 4.0 * (double)d * (m + 2), reinterpret_cast<hipStream_t>(stream));
  ZENO_TRY(launch_krum(G, ldg, m, d, b, out, chosen, krum_scores, workspace, reinterpret_cast<hipStream_t>(stream)));
  return ZENO_OK;
}

const char* zeno_status_string(int32_t status) {
  switch (status) {
    case ZENO_OK: return "ok";
    case ZENO_ERR_INVALID_ARG: return "invalid argument";
    case ZENO_ERR_UNSUPPORTED: return "unsupported size";
    case ZENO_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ZENO_ERR_DEVICE: return "HIP launch failed";
    case ZENO_ERR_HOST_MEMORY: return "out of host memory";
  }
  return "unknown status";
}

}  // extern "C"
