/*
 * ens.h - C interface of the MI355X ensemble-inference library.
 *
 * The library implements the hot path of an inference system for ensembles of
 * deep neural networks (arxiv 2208.14049): the batched forward pass of every
 * ensemble member co-located on one GPU and the averaging combination rule,
 * laid out by an allocation matrix that a host-side optimizer chooses.
 *
 * Conventions
 *   - Every function returns ENS_OK (0) or a negative ens_status; nothing throws
 *     across this boundary.  ens_strerror() names a status.
 *   - Pointers are HOST pointers unless the comment says "device".
 *   - The caller owns every buffer it passes in; the library owns the handle and
 *     everything reachable from it (weights, activation arenas, streams).
 *   - A handle is not thread-safe; ens_predict / ens_bench are synchronous.
 *   - All image tensors are NHWC (channels fastest).
 */
#ifndef ENS_H
#define ENS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ENS_OK = 0,
    ENS_E_INVALID = -1,     /* malformed description, matrix or argument                      */
    ENS_E_NOMEM = -2,       /* a member or worker does not fit in device memory: the paper's
                               "{-1, None, None}" message, section "The prediction accumulator" */
    ENS_E_NOFIT = -3,       /* Algorithm 1: no device has enough memory for a member           */
    ENS_E_HIP = -4,         /* a HIP runtime call failed                                       */
    ENS_E_NODEVICE = -5,    /* no GPU visible                                                  */
    ENS_E_UNSUPPORTED = -6, /* description uses a shape the GPU kernels do not cover           */
    ENS_E_TOOBIG = -7       /* ens_predict_static: the request does not fit the static scratch */
} ens_status;

/* ---- member description --------------------------------------------------------------------
 * A member is a list of operations over numbered NHWC tensors (tensor 0 is the input image at
 * the member's own resolution) and one flat fp32 parameter blob.  Semantics of each operation:
 *   CONV     dst[.., dst_c0:+cout] = act(bn(conv(pre(src[.., src_c0:+cin])) + bias) + res)
 *            weights [kh][kw][cin][cout] at off_w; zero padding, pt rows above and pl columns
 *            to the left; output size = the dst tensor's H x W; `pre` applies an inference
 *            batch-norm (off_pre) then ReLU to the in-bounds input values; with r = g > 1 the
 *            convolution has g groups: output channel co sees the input channels of group
 *            co / (cout/g) only and the weights are [kh][kw][cin/g][cout] (bf16 members, cout/g a
 *            divisor or a multiple of 32, no `pre`: otherwise ENS_E_UNSUPPORTED);
 *   DWCONV   depthwise, weights [kh][kw][c];
 *   MAXPOOL / AVGPOOL  over the in-bounds part of the window;
 *   GAP      mean over all pixels (of relu(bn(x)) when pre);
 *   FC       dst = src . W[cin][cout] + bias, src a 1 x 1 x cin tensor;
 *   SE       squeeze-excite: s = mean over pixels, g = sigmoid(W2^T silu(W1^T s + b1) + b2),
 *            dst = src * g; W1 [c][r] at off_w, b1 at off_b, W2 [r][c] at off_w2, b2 at off_b2.
 * Batch-norm parameters are four consecutive vectors [gamma, beta, mean, var], eps = 1e-5.
 * Offsets are in floats into the blob; -1 = absent.
 */
enum { ENS_OP_CONV = 1, ENS_OP_DWCONV = 2, ENS_OP_MAXPOOL = 3, ENS_OP_AVGPOOL = 4,
       ENS_OP_GAP = 5, ENS_OP_FC = 6, ENS_OP_SE = 7 };
enum { ENS_ACT_NONE = 0, ENS_ACT_RELU = 1, ENS_ACT_SILU = 2 };
enum { ENS_FP32 = 0, ENS_BF16 = 1 };

typedef struct { int32_t h, w, c; } ens_tensor;

typedef struct {
    int32_t kind, src, src_c0, cin, dst, dst_c0, cout;
    int32_t kh, kw, sh, sw, pt, pl, act, res, res_c0, pre, r;
    int64_t off_w, off_b, off_bn, off_pre, off_w2, off_b2;
} ens_op;

/* How to draw one parameter tensor from a seed (used when ens_member_spec.params is NULL). */
enum { ENS_PARAM_WEIGHT = 1, ENS_PARAM_BIAS = 2, ENS_PARAM_BN = 3 };
typedef struct {
    int32_t role;      /* ENS_PARAM_*                                                        */
    int32_t channels;  /* BN: channel count (size = 4 * channels)                            */
    int64_t offset;    /* in floats into the blob                                            */
    int64_t size;      /* in floats                                                          */
    double  scale;     /* WEIGHT: standard deviation; BN: the constant gamma; BIAS: unused   */
} ens_param;

typedef struct {
    const ens_tensor* tensors;  int32_t n_tensors;
    const ens_op*     ops;      int32_t n_ops;
    int32_t out_tensor;         /* the 1 x 1 x classes tensor holding the logits             */
    int32_t dtype;              /* ENS_FP32: fp32 storage and arithmetic;
                                   ENS_BF16: bf16 storage, fp32 accumulation                 */
    const float* params;        /* host, n_params floats; NULL = draw from the seed          */
    int64_t n_params;
    const ens_param* param_specs; int32_t n_param_specs;   /* needed only when params == NULL */
} ens_member_spec;

/* ---- allocation matrix ---------------------------------------------------------------------
 * Section "The allocation matrix data structure": rows are devices, columns are DNNs, 0 = no
 * worker, any other value = that worker's batch size; a column of zeros is illegal.  On one
 * GPU the rows are instance slots that share the GPU's memory.
 */
#define ENS_MAX_SLOTS   16
#define ENS_MAX_MEMBERS 64
#define ENS_MAX_DOMAIN  16

typedef struct {
    int32_t rows, cols;
    int32_t batch[ENS_MAX_SLOTS][ENS_MAX_MEMBERS];
    int64_t bytes;      /* out: device memory the matrix needs (weights + arenas)             */
    double  score;      /* out: images per second measured for it, 0 if never benchmarked     */
    int32_t n_bench;    /* out: number of benchmarks the optimizer ran                        */
} ens_alloc;

typedef struct {
    int32_t n_domain;  int32_t domain[ENS_MAX_DOMAIN]; /* batch sizes, default {8,16,32,64,128} */
    int32_t default_batch;      /* Algorithm 1 places every member at this size, default 8     */
    int32_t segment_size;       /* default 128; raised to the largest batch size if smaller    */
    int32_t max_neighs;         /* default 100                                                 */
    int32_t max_iter;           /* moves of Algorithm 2, default 10; raised to (slots - members) when
                                   that is larger (section "Offline benchmark settings")       */
    int32_t slots;              /* instance slots (rows) on the GPU, default 1                 */
    int32_t strategy;           /* 0 = Algorithm 1 then Algorithm 2; 1 = Algorithm 1 only;
                                   2 = BBS baseline (each member's batch size tuned alone)     */
    uint64_t seed;              /* seeds the draw of neighbours                                */
    int64_t n_calib;            /* calibration images per benchmark, default 1024              */
    int32_t repeats;            /* timed repetitions per benchmark (median), default 3         */
    int32_t verbose;            /* non-zero: one line per benchmark on stderr (a plan over many
                                   members runs for minutes)                                   */
} ens_plan_opts;

typedef struct ens_handle ens_handle;

/* ---- life cycle ----------------------------------------------------------------------------
 * ens_load: section "Inference frameworks" ("load" puts a trained DNN on a device).  Turns every
 * batch-norm into a scale and a bias per output channel (fp32 members: the scale goes into the
 * weights; bf16 members keep the weights as given and apply the fp32 scale to the sum), converts
 * to the member's dtype and uploads.  Parameters
 * come from spec.params, or are drawn from `seed` (member index, parameter index) with the
 * library's counter-based generator when spec.params is NULL.  On ENS_E_NOMEM nothing stays
 * allocated.  *out is the new handle.
 */
int ens_load(const ens_member_spec* specs, int32_t n_members, uint64_t seed, ens_handle** out);
void ens_free(ens_handle* h);

/* Input geometry and buffer placement for ens_predict: requests are n x base_h x base_w x 3
 * fp32 images; members whose own resolution differs are fed a bilinear resize (half-pixel
 * centres, edge clamp).  images_on_device / probs_on_device: the pointers given to ens_predict
 * are device pointers.  Default: base size = member 0's input size, host pointers.
 * Device buffers are read and written on the library's own streams, which are not ordered against
 * any stream of the caller: the images must be complete in device memory before ens_predict is
 * called (synchronise the producing stream first), and the probabilities are complete when it
 * returns. */
int ens_set_io(ens_handle* h, int32_t base_h, int32_t base_w, int32_t images_on_device,
               int32_t probs_on_device);

/* ---- allocation ----------------------------------------------------------------------------
 * ens_plan: section "The allocation optimizer".  Algorithm 1 (worst-fit-decreasing) places every
 * member at default_batch within mem_budget_bytes, Algorithm 2 (bounded greedy) then benchmarks
 * neighbouring matrices on calibration images; the result is installed and returned.
 * opts == NULL takes the paper's settings.  ENS_E_NOFIT if a member fits nowhere.
 */
int ens_plan(ens_handle* h, uint64_t mem_budget_bytes, const ens_plan_opts* opts, ens_alloc* out);

/* Installs a caller-made matrix, or one kept from an earlier ens_plan (section "The allocation
 * optimizer" keeps the best matrix for reuse).  ENS_E_INVALID for a zero column or a non-positive size, ENS_E_NOMEM when the
 * workers do not fit.  Builds one stream and one activation arena per non-zero cell. */
int ens_set_alloc(ens_handle* h, const ens_alloc* a, int32_t segment_size);

/* "Benchmark Mode" of section "The inference system": installs `a`, predicts n_calib synthetic
 * calibration images resident on the device and returns images per second (median of `repeats`
 * runs after one warm-up); *img_per_sec = 0 when a worker does not fit in memory. */
int ens_bench(ens_handle* h, const ens_alloc* a, int32_t segment_size, int64_t n_calib,
              int32_t repeats, double* img_per_sec);

/* ---- prediction ----------------------------------------------------------------------------
 * "Deploy Mode" of section "The inference system", f(X, A) -> Y: the request is cut into
 * segments (section "The segment ids broadcaster"), every segment goes once to every member,
 * a member's workers cut segments into batches of their own size (section "The worker pool"),
 * and Y[i] = sum_m softmax(logits_m[i]) / M (section "The prediction accumulator").
 *   images   : n x base_h x base_w x 3 fp32 (host or device, see ens_set_io)
 *   probs_out: n x classes fp32, written completely before the call returns
 * Needs an installed allocation (ens_plan or ens_set_alloc); without one, every member gets one
 * worker of batch size 8.  A call with a larger n than any before it (or with another device
 * image pointer) allocates device memory and rewrites argument blocks before it starts;
 * ens_predict_static below never allocates.
 */
int ens_predict(ens_handle* h, const float* images, int64_t n, float* probs_out);

/* ens_predict for callers that cannot allocate device memory (code under HIP graph capture set-up,
 * tight serving loops, harnesses that forbid hipMalloc): the same computation as ens_predict with
 * the per-request scratch of the call (the members' logits, members x n x classes fp32, and the
 * device table of their pointers), which ens_predict grows with hipMalloc, placed in a fixed device
 * array inside the library (ens_static_scratch_bytes() bytes, 32 MiB, held by every GPU the
 * library is loaded on until the process ends).  The call allocates and frees nothing.
 *   d_images   : DEVICE, n x base_h x base_w x 3 fp32, complete before the call
 *   d_probs_out: DEVICE, n x classes fp32, complete when the call returns
 * Needs an installed allocation (ens_plan / ens_set_alloc: they allocate the workers' arenas) and
 * per-kernel profiling switched off; ENS_E_INVALID otherwise.  ENS_E_TOOBIG, with a message on
 * stderr, when members x n x classes x 4 bytes exceed the array less its 4 KiB table (3 members of
 * 1000 classes: n <= 2795).  The array is shared by every handle and call on a GPU and keeps the last
 * call's contents; a call writes every value it later reads, so nothing needs clearing, but calls
 * that overlap in time on one GPU race.  ens_member_logits reads the array after such a call. */
int ens_predict_static(ens_handle* h, const float* d_images, int64_t n, float* d_probs_out);
int ens_static_scratch_bytes(void);

/* Combination rule of ens_predict (section "The prediction accumulator").  The default is the
 * paper's: the mean of the members' softmax outputs.  The same section names two more:
 *   ENS_COMBINE_WEIGHTED  Y[i] = sum_m weights[m] * softmax(logits_m[i]); weights: n_members host
 *                         floats, copied by the call and used as given (not normalised)
 *   ENS_COMBINE_VOTE      majority voting: Y[i, c] = (members whose arg-max for sample i is c) / M,
 *                         lowest class on exact ties; weights is ignored
 * ENS_E_INVALID for an unknown rule or missing weights. */
enum { ENS_COMBINE_MEAN = 0, ENS_COMBINE_WEIGHTED = 1, ENS_COMBINE_VOTE = 2 };
int ens_set_combination(ens_handle* h, int32_t rule, const float* weights);

/* Overhead experiment of section "Overhead of the inference system": with the fake predictor on,
 * every member's forward pass (input staging included) is replaced by a prediction of zeros; the
 * partition into segments and batches, the workers' streams, the event join and the combination
 * rule still run.  The wall time of such an ens_predict is the system's own overhead. */
int ens_debug_fake_predictor(ens_handle* h, int32_t on);

/* Last per-member logits of the most recent ens_predict (n x classes fp32, host destination);
 * for tests of single members. */
int ens_member_logits(ens_handle* h, int32_t member, int64_t n, float* logits_out);

/* Copies tensor `tensor` of member `member` as worker 0 of that member last computed it
 * (first `n_images` images of its last batch) to `out` as fp32 NHWC, logical channels only.
 * For tests of single layers.  A worker's arena reuses the memory of tensors that are no
 * longer needed; ens_debug_keep_tensors(h, 1) before the allocation is installed gives every
 * tensor its own region so that all of them can be read back. */
int ens_debug_keep_tensors(ens_handle* h, int32_t on);
int ens_debug_tensor(ens_handle* h, int32_t member, int32_t tensor, int32_t n_images, float* out);

/* ---- queries -------------------------------------------------------------------------------*/
int ens_classes(const ens_handle* h);
int ens_n_members(const ens_handle* h);
/* Device bytes of member m: weights (once per member) and the activation arena of one worker
 * at the given batch size (peak live activations by liveness analysis of the operation list). */
int ens_member_bytes(const ens_handle* h, int32_t member, int32_t batch, int64_t* weight_bytes,
                     int64_t* arena_bytes);
/* Same figures from a description alone; host-only, needs no GPU. */
int ens_spec_bytes(const ens_member_spec* spec, int32_t batch, int64_t* weight_bytes,
                   int64_t* arena_bytes);
/* Per-kernel timing.  With profiling on, every kernel launch of ens_predict / ens_bench carries
 * a pair of HIP events attached to its dispatch (stamped with the kernel's own begin and end), and
 * the durations are summed per kernel class after the call.  ens_profile_get enumerates the classes of the last call
 * (idx = 0, 1, ...; ENS_E_INVALID past the end): name, summed milliseconds, launches, the
 * algorithmic flop and the algorithmic bytes (each input, weight and output read or written
 * once) of those launches.  ens_last_ms is the wall time of the last ens_predict. */
int ens_set_profiling(ens_handle* h, int32_t on);
/* Measurement aid: with one_stream on, every worker issues its kernels on one stream, so that each kernel
 * has the GPU to itself and ens_profile_get reports durations that no co-running kernel stretches.  Same
 * results, no overlap; not for serving. */
int ens_debug_one_stream(ens_handle* h, int32_t on);
int ens_profile_get(const ens_handle* h, int32_t idx, char* name, int32_t name_len, double* ms,
                    int64_t* launches, double* flop, double* bytes);
double ens_last_ms(const ens_handle* h);

/* ---- host-only planner (no GPU needed) -------------------------------------------------------
 * The optimizer of section "The allocation optimizer" over an explicit memory model and an
 * explicit benchmark callback, for any number of devices.  A pool holds, for each member with
 * a worker in it, the member's weights once plus one arena per worker.
 */
typedef struct {
    int32_t n_models, n_rows, n_pools, n_domain;
    const int32_t* domain;        /* n_domain batch sizes                                      */
    int32_t default_batch;        /* must be in the domain                                     */
    const int64_t* weight_bytes;  /* n_models                                                  */
    const int64_t* arena_bytes;   /* n_models x n_domain                                       */
    const int32_t* row_pool;      /* n_rows: pool of each row                                  */
    const int32_t* row_is_gpu;    /* n_rows: 1 = GPU, 0 = CPU (Algorithm 1 prefers GPUs)       */
    const int64_t* pool_cap;      /* n_pools                                                   */
    int32_t max_iter, max_neighs;   /* max_iter is raised to n_rows - n_models when that is larger */
    uint64_t seed;
} ens_plan_problem;

typedef double (*ens_bench_fn)(const int32_t* matrix /* n_rows x n_models */, void* user);
typedef double (*ens_bench_single_fn)(int32_t model, int32_t batch, void* user);

int ens_planner_fit_mem(const ens_plan_problem* p, const int32_t* matrix);           /* 1 / 0 */
int ens_planner_wfd(const ens_plan_problem* p, int32_t* matrix_out);                 /* Algorithm 1 */
int ens_planner_neighbors(const ens_plan_problem* p, const int32_t* matrix, int32_t* out,
                          int32_t max_out, int32_t* n_out);      /* valid matrices one cell away */
int ens_planner_greedy(const ens_plan_problem* p, int32_t* matrix_inout, ens_bench_fn bench,
                       void* user, double* score, int32_t* n_bench);                 /* Algorithm 2 */
int ens_planner_bbs(const ens_plan_problem* p, ens_bench_single_fn bench, void* user,
                    int32_t* batch_out, int32_t* n_bench);                           /* BBS baseline */
/* Segment / batch partition of a request: writes up to max_out (start, end) pairs. */
int ens_partition(int64_t nb_images, int32_t segment_size, int32_t batch, int64_t* starts,
                  int64_t* ends, int32_t max_out, int32_t* n_out);

/* Hand-out of a member's segments among its n_workers workers (section "Data-parallelism": the
 * workers of one DNN take segment ids from the same FIFO queue, so each gets segments in proportion to
 * its speed).  The queue is run in estimated time on the host: a worker of batch size b needs
 * ceil(L / b) * launch_cost + L * image_cost for a segment of L images, and each segment, in order,
 * goes to the worker that becomes free first (lowest index on ties).  Writes the owner of each of the
 * first max_out segments, *n_out = number of segments. */
int ens_hand_out(int64_t nb_images, int32_t segment_size, const int32_t* batch, int32_t n_workers,
                 double launch_cost, double image_cost, int32_t* owner_out, int32_t max_out, int32_t* n_out);

const char* ens_strerror(int status);
const char* ens_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ENS_H */
