/*
 * zeno.h -- C ABI of the MI355X (gfx950) Zeno aggregation library.
 *
 * The library implements the server-side aggregation step of
 * "Zeno: Distributed Stochastic Gradient Descent with Suspicion-based
 * Fault-tolerance" (arXiv 1805.10032):
 *
 *   Definition 2 (Stochastic Descendant Score)
 *       Score_{gamma,rho}(u, x) = f_r(x) - f_r(x - gamma u) - rho ||u||^2,
 *       f_r = mean loss over the n_r samples the server drew for this iteration.
 *   Definition 3 (Suspicion-based Aggregation, Zeno_b)
 *       average of the m-b candidates with the highest scores.
 *   Section 6.1.1 baselines: Mean, and Definition 4 (marginal Median).
 *
 * Conventions shared by every call
 * --------------------------------
 * Pointers.  Arguments marked DEVICE point to HIP device memory of the current
 *   device, owned by the caller, at least 4-byte aligned.  Arguments marked
 *   HOST are ordinary host pointers and are read before the call returns.
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default
 *   stream).  Every call only enqueues work on that stream and returns; no call
 *   synchronises with the host, reads device results on the host, or allocates
 *   or frees device memory.  Scratch memory is the caller's `workspace`.
 * Parameter layout.  A parameter vector of the model (x, and every row of the
 *   candidate matrix G) is, for l = 1..L: the weight matrix W_l stored
 *   row-major as [dims[l] x dims[l-1]] (out x in), followed, if has_bias, by
 *   the bias b_l[dims[l]].  d = zeno_model_num_params().
 * Candidate matrix.  G is [m x d] row-major; consecutive rows are ldg >= d
 *   floats apart (ldg = d: densely packed).  Neither d nor ldg need be a
 *   multiple of 4, so rows may be only 4-byte aligned and every kernel accepts
 *   that.  The server decides where the workers' vectors land, and the layout
 *   the kernels are fastest on is G 128-byte aligned with ldg an ODD multiple of
 *   32 floats: then every 128-byte memory line of a row belongs to one load
 *   instruction, the rows are streamed with loads that bypass cache retention,
 *   and the rows of different candidates start on different halves of a 256-byte
 *   span (an even multiple measures about 2 % slower on multi-gigabyte G).
 *   A densely packed G whose rows are 16-byte aligned (G 16-byte aligned, d a
 *   multiple of 4) comes within 4 % of that in zeno_score with the bf16 forward
 *   pass on layers whose input width is a multiple of 64: their weight tiles
 *   are loaded on a column grid shifted to the lines of each candidate's rows.
 * Errors.  Every call returns a zeno_status_t; nothing is thrown across the
 *   ABI.  Argument errors are detected on the host before anything is
 *   enqueued, so a failed call leaves the outputs untouched.
 * Non-finite data.  "Arbitrary values" (Section 3, Eq. 1) include NaN/Inf
 *   rows: they propagate through the forward pass, a NaN score ranks as
 *   -infinity, ties go to the lower index, and the median sorts NaN above +Inf.
 */
#ifndef ZENO_H_
#define ZENO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZENO_MAX_LAYERS 8
#define ZENO_MAX_CANDIDATES 1024

typedef enum {
  ZENO_OK = 0,
  ZENO_ERR_INVALID_ARG = 1, /* NULL/misaligned pointer, m<1, m>1024, b<0, b>=m, n_r<1, ldg<d, bad gamma/rho/dims */
  ZENO_ERR_UNSUPPORTED = 2, /* a size beyond what the kernels cover (see each call) */
  ZENO_ERR_WORKSPACE = 3,   /* workspace NULL, misaligned (256 B) or smaller than the query says */
  ZENO_ERR_DEVICE = 4,      /* a HIP launch failed */
  ZENO_ERR_HOST_MEMORY = 5  /* the host-side model object could not be allocated */
} zeno_status_t;

typedef enum {
  ZENO_LOSS_SQUARED = 0,   /* f(x; (a, y)) = 1/2 (model(a) - y)^2, output width 1 */
  ZENO_LOSS_SOFTMAX_CE = 1 /* f(x; (a, y)) = logsumexp(model(a)) - model(a)[y], natural log */
} zeno_loss_t;

typedef enum {
  ZENO_FWD_FP32 = 0, /* forward-pass products in fp32 (fp32 matrix cores), fp32 accumulate */
  ZENO_FWD_BF16 = 1  /* matrix operands rounded to bf16, fp32 accumulate */
} zeno_fwd_dtype_t;

/* Model whose loss the score evaluates: L linear layers, ReLU between them,
 * none after the last.  HOST struct, copied by zeno_model_create. */
typedef struct {
  int32_t n_layers;                  /* L, 1..ZENO_MAX_LAYERS */
  int32_t dims[ZENO_MAX_LAYERS + 1]; /* dims[0] = input width ... dims[L] = output width, each >= 1 */
  int32_t has_bias;                  /* 0 or 1 */
  int32_t loss;                      /* zeno_loss_t; ZENO_LOSS_SQUARED requires dims[L] == 1 */
  int32_t fwd;                       /* zeno_fwd_dtype_t */
} zeno_model_desc_t;

typedef struct zeno_model zeno_model_t; /* opaque HOST object owned by the library */

/* The n_r samples the server drew for this iteration (Algorithm 1, server
 * side: drawn after the candidates arrived; one batch for all m candidates). */
typedef struct {
  int32_t n_r;             /* >= 1 */
  const float* features;   /* DEVICE [n_r x dims[0]] row-major */
  const int32_t* labels;   /* DEVICE [n_r], softmax-CE only, 0 <= label < dims[L]; a label outside that
                              range makes every score NaN (nothing is read out of bounds) */
  const float* targets;    /* DEVICE [n_r], squared loss only */
} zeno_batch_t;

/* Create / destroy the host-side model object.  `out` receives the handle.
 * Errors: INVALID_ARG for NULL pointers, n_layers or dims out of range, a
 * squared loss with output width != 1, unknown enum values. */
zeno_status_t zeno_model_create(const zeno_model_desc_t* desc, zeno_model_t** out);
void zeno_model_destroy(zeno_model_t* model);

/* Convolutional model (Section 6.1 evaluates Zeno on a network of four convolutional layers and one
 * fully connected layer; the paper gives no widths, so they are the caller's): n_conv convolutions
 * with 3 x 3 kernels, zero padding 1 and stride 1 or 2, ReLU after each, then one fully connected
 * layer on the flattened last map, no activation.  Images and maps are NHWC; a map shrinks to
 * (h - 1) / stride + 1 rows (integer division), likewise columns.
 * Parameter layout of x and of every row of G: for every convolution the kernel
 * W[c_out][ky][kx][c_in] row-major followed, if has_bias, by bias[c_out]; then the fully connected
 * W[fc_out][h * w * c], whose input is the last map flattened in (y, x, c) order, and its bias.
 * The batch's features are the images, [n_r x in_h * in_w * in_c].
 * Forward passes run in fp32 on the fp32 matrix cores; batches of more than 128 samples are
 * UNSUPPORTED by zeno_score for these models.  HOST struct, copied by zeno_cnn_model_create. */
#define ZENO_MAX_CONV 8
typedef struct {
  int32_t in_h, in_w, in_c;            /* each >= 1 */
  int32_t n_conv;                      /* 1..ZENO_MAX_CONV */
  int32_t conv_c[ZENO_MAX_CONV];       /* output channels of every convolution, >= 1 */
  int32_t conv_stride[ZENO_MAX_CONV];  /* 1 or 2 */
  int32_t fc_out;                      /* output width, >= 1 */
  int32_t has_bias;                    /* 0 or 1 */
  int32_t loss;                        /* zeno_loss_t; ZENO_LOSS_SQUARED requires fc_out == 1 */
} zeno_cnn_desc_t;

/* Handle for a convolutional model; used with zeno_score, zeno_score_static, zeno_model_num_params,
 * zeno_score_workspace_bytes and zeno_model_destroy like the handle of zeno_model_create.
 * Errors: INVALID_ARG for NULL pointers or fields out of range. */
zeno_status_t zeno_cnn_model_create(const zeno_cnn_desc_t* desc, zeno_model_t** out);

/* d, the length of a parameter vector in the layout above. */
int64_t zeno_model_num_params(const zeno_model_t* model);

/* Bytes of DEVICE scratch that zeno_score needs for m candidates and a batch of
 * n_r samples (activations of the m+1 forward passes, partial norms).  Returns
 * 0 for invalid arguments. */
size_t zeno_score_workspace_bytes(const zeno_model_t* model, int32_t m, int32_t n_r);

/* Definition 2 for every row of G:
 *   scores[i] = f_r(x) - f_r(x - gamma G[i]) - rho ||G[i]||^2,  i = 0..m-1.
 * f_r(x) is evaluated once and shared (Section 6.7: (m+1) loss evaluations).
 * The perturbed parameters x - gamma G[i] are never materialised: each row of
 * G is read from memory once, and what is propagated through the layers is the
 * change of the activations relative to the forward pass at x, so that the
 * difference f_r(x) - f_r(x - gamma u) is formed without cancellation.
 *   x       DEVICE [d]            current parameters
 *   G, ldg  DEVICE [m x d], rows ldg >= d floats apart: candidate gradient estimators, 1 <= m <= 1024
 *   batch   HOST struct with DEVICE pointers
 *   gamma   learning rate, finite, >= 0;  rho  finite, >= 0 (rho = 0 is the
 *           appendix's choice for mu >= 0)
 *   scores  DEVICE [m] fp32 out
 *   workspace DEVICE, 256-byte aligned, >= zeno_score_workspace_bytes(model, m, n_r)
 * Batches of more than 128 samples are processed in passes of 128, each pass
 * reading G again. */
zeno_status_t zeno_score(const zeno_model_t* model, const float* x, const float* G, int64_t ldg, int32_t m,
                         const zeno_batch_t* batch, float gamma, float rho, float* scores,
                         void* workspace, size_t workspace_bytes, void* stream);

/* zeno_score for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as zeno_score, bit for bit, but the scratch is a static device
 * array inside the library (ZENO_STATIC_SCRATCH_BYTES per GPU, held until the process ends), so
 * the call allocates nothing, frees nothing and takes no workspace.
 *   UNSUPPORTED if zeno_score_workspace_bytes(model, m, n_r) exceeds ZENO_STATIC_SCRATCH_BYTES
 *     (32 MiB covers e.g. a 3072->512->10 model with m = 20, or the paper's m = 20, n_r = 4 on
 *     far larger models; it does not cover hundreds of candidates on 2048-wide layers);
 *   DEVICE if the array's address cannot be obtained on the current device.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race and give wrong scores; calls on one stream are ordered and safe.  The array
 * keeps the previous call's contents; no call depends on them. */
#define ZENO_STATIC_SCRATCH_BYTES (32u << 20)
zeno_status_t zeno_score_static(const zeno_model_t* model, const float* x, const float* G, int64_t ldg, int32_t m,
                                const zeno_batch_t* batch, float gamma, float rho, float* scores, void* stream);

/* Definition 3: out = (1/(m-b)) * sum of the m-b rows of G with the highest
 * scores, 0 <= b < m (b = 0 is the Mean).  The selection runs on the device
 * from `scores` (no host round trip); rows are summed in ascending index order
 * in fp64 and rounded once to fp32.
 *   scores   DEVICE [m] (as written by zeno_score)
 *   out      DEVICE [d]
 *   selected DEVICE [m-b] int32 out, ascending indices of the chosen rows; may be NULL */
zeno_status_t zeno_aggregate(const float* G, int64_t ldg, const float* scores, int32_t m, int64_t d, int32_t b,
                             float* out, int32_t* selected, void* stream);

/* Definition 3 followed by the server's update of Algorithm 1 in the same pass over
 * the chosen rows:  x_next = x - gamma * Zeno_b(G).  The step is taken from the
 * float64 average before it is rounded (x_next[j] = fl32(x[j] - gamma * avg_j), product
 * and difference in float64), so it costs one read of x and one write of x_next
 * instead of a separate pass over d values.
 *   x       DEVICE [d]   current parameters
 *   x_next  DEVICE [d]   out; may be x itself (in place)
 *   out     DEVICE [d]   the aggregate as zeno_aggregate writes it, or NULL if only x_next is wanted
 *   gamma   finite, >= 0
 * Other arguments and errors as for zeno_aggregate. */
zeno_status_t zeno_aggregate_update(const float* G, int64_t ldg, const float* scores, int32_t m, int64_t d,
                                    int32_t b, float gamma, const float* x, float* x_next, float* out,
                                    int32_t* selected, void* stream);

/* Mean baseline (Section 6.1.1): out[j] = (1/m) sum_i G[i][j]. */
zeno_status_t zeno_mean(const float* G, int64_t ldg, int32_t m, int64_t d, float* out, void* stream);

/* Marginal median (Definition 4): out[j] = median_i G[i][j]; for even m the
 * midpoint of the two middle values (formed in float64, rounded once).  NaN entries
 * sort above +inf.  Up to m = 128 the values of a column are sorted in registers; for
 * 128 < m <= 1024 the median is found by rank selection on keys kept in LDS, which is
 * several times slower per byte of G. */
zeno_status_t zeno_median(const float* G, int64_t ldg, int32_t m, int64_t d, float* out, void* stream);

/* Krum_b (Definition 5, the paper's main baseline): out = the row of G whose sum of squared
 * distances to its m-b-2 nearest other rows is smallest (ties: lower index).  The distances
 * come from the Gram matrix G G^T, taken in one pass over G on the bf16 matrix cores (every
 * float split into three bf16 pieces, six piece products: float32 accuracy) and summed in
 * float64, as S_ii + S_jj - 2 S_ij; they are exact to about 1e-5 of ||G_i||^2 + ||G_j||^2.  When a
 * distance that enters a score is below 1e-3 of that scale (rows much closer to each other than to
 * the origin), a second pass over G repeats the computation on the rows minus the row the first
 * pass chose, which makes the distances around that row exact to about 1e-5 of themselves; the
 * decision is taken on the device and costs nothing when it is not needed.  Two rows whose Krum
 * scores differ by less than these errors may be chosen either way.  Requires
 * m - b - 2 >= 1; UNSUPPORTED for m > 128.  A row that holds NaN or Inf is at infinite distance
 * from every row: it is nobody's near neighbour and its own score is +infinity.
 *   out         DEVICE [d]    copy of the chosen row
 *   chosen      DEVICE [1]    int32 out, index of the chosen row
 *   krum_scores DEVICE [m]    out, the m sums of squared distances, or NULL
 *   workspace   DEVICE, 256-byte aligned, >= zeno_krum_workspace_bytes(m) */
size_t zeno_krum_workspace_bytes(int32_t m);
zeno_status_t zeno_krum(const float* G, int64_t ldg, int32_t m, int64_t d, int32_t b, float* out, int32_t* chosen,
                        float* krum_scores, void* workspace, size_t workspace_bytes, void* stream);

/* Text of a status code; any other value gives "unknown status". */
const char* zeno_status_string(int32_t status);

/* Host-only self-check of the scratch layout of zeno_score (Definition 2's m+1 forward passes keep
 * their activations there): walks the launch sequence for (model, m, n_r) without touching a
 * device and verifies, for every workgroup width a launch may take, that everything the launch
 * writes lies inside its slot of the workspace.  OK, INVALID_ARG for bad arguments, WORKSPACE if a
 * launch would leave its slot (a bug in the library: zeno_score makes the same check for the
 * widths it really uses and then enqueues nothing).  UNSUPPORTED for convolutional models. */
zeno_status_t zeno_score_plan_check(const zeno_model_t* model, int32_t m, int32_t n_r);

/* Per-launch timing, a measurement aid (Section 5.3 prices the step by its
 * O(d m) passes over the candidates; this reports what each pass costs).
 * While enabled, every kernel launch of the library is bracketed by a pair of
 * HIP events recorded on the launch's own stream.  zeno_profile_collect waits
 * for the recorded events, copies up to max_records records (in launch order)
 * into the HOST array `records`, returns how many it wrote and forgets them
 * all.  algorithmic_bytes is what the launch must move by definition: the
 * layer block of every source it streams, or the rows read plus the row
 * written for the aggregators.  Not thread-safe against concurrent launches
 * of the same process beyond a mutex around the record list. */
typedef enum {
  ZENO_KERNEL_PACK = 0,       /* batch features into matrix-operand order */
  ZENO_KERNEL_LAYER_BASE = 1, /* one layer of the pass at x */
  ZENO_KERNEL_LAYER_CAND = 2, /* one layer of the m candidate passes (streams G) */
  ZENO_KERNEL_LOSS = 3,       /* per-sample loss differences */
  ZENO_KERNEL_COMBINE = 4,    /* mean, norm and the three-term score */
  ZENO_KERNEL_AVERAGE = 5,    /* selection + average of the chosen rows */
  ZENO_KERNEL_MEAN = 6,
  ZENO_KERNEL_MEDIAN = 7,
  ZENO_KERNEL_AVERAGE_UPDATE = 8, /* selection + average + x_next = x - gamma * average */
  ZENO_KERNEL_KRUM = 9,           /* Gram matrix + selection + copy of the chosen row */
  ZENO_KERNEL_CONV_BASE = 10,     /* one convolution of the pass at x */
  ZENO_KERNEL_CONV_CAND = 11,     /* one convolution of the m candidate passes */
  ZENO_KERNEL_AUX = 12            /* fills, squared norms of the convolution kernels */
} zeno_kernel_t;

typedef struct {
  int32_t kernel; /* zeno_kernel_t */
  int32_t layer;  /* 0-based layer index for the layer kernels, else 0 */
  float ms;       /* elapsed time between the two events */
  double algorithmic_bytes;
  /* layer kernels only (else 0): the launch shape that ran */
  int32_t waves;      /* waves per workgroup that own different 32-feature tiles: 1, 4 or 8 */
  int32_t k_split;    /* waves that share one feature tile and split the input width: 1, 2 or 4 */
  int32_t streaming;  /* 1: rows read with non-temporal loads (line-aligned layout), 0: plain loads,
                         2: non-temporal loads on a column grid shifted to the lines of each candidate's rows
                            (16-byte aligned dense rows, bf16 forward), 3: the same for rows that are only 8-byte
                            aligned (d mod 4 = 2) */
  int32_t row_blocks; /* 32-sample accumulator blocks per wave: 1, 2 or 4 */
  int32_t merged;     /* 1: the launch carries the candidates' layer AND the pass at x through another layer */
  int32_t second;     /* 1: candidates with the second matrix product (layers after the first) */
  int32_t k_slices;   /* workgroups that share one feature tile and split the input width: 1..8 (launches of one-wave
                         tiles: every tile; eight-wave launches: the tiles of the sliced tail, see tail_candidates) */
  int32_t candidates;      /* candidate launches: the rows of G the launch streams */
  int32_t tail_candidates; /* eight-wave launches: the last so many candidates' tiles (and the pass at x, if merged)
                              ran as k_slices K slices each at the end of the launch; 0: none */
} zeno_profile_record_t;

zeno_status_t zeno_profile_enable(int32_t enable);
int32_t zeno_profile_collect(zeno_profile_record_t* records, int32_t max_records);

#ifdef __cplusplus
}
#endif
#endif /* ZENO_H_ */
