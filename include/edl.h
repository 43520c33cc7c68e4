/*
 * edl.h - C boundary of the data-parallel training step of an elastic
 * deep-learning job, native on MI355X (gfx950).
 *
 * One handle is one job on one GPU.  The p workers of the job are simulated
 * as p shards of the aggregate mini-batch, processed one after the other on
 * the handle's stream.  What the calls mean, in the paper's terms:
 *
 *   edl_init      init() of the framework API (section 3.2, Table 1)
 *   edl_shard     elastic_shard_generator().next() (sections 3.2, 4.3)
 *   edl_step      one mini-batch: session.run(obj) + all_reduce() +
 *                 notify_batch_end() (section 3.2); a p that differs from the
 *                 previous call's is a scale_in / scale_out that takes effect
 *                 at this mini-batch boundary (sections 3.1, 4.2)
 *   edl_snapshot  the model a joining worker receives from one existing
 *                 worker (section 4.2), with the job meta-data a new leader
 *                 receives (section 4.2, scale in) and the data-loading
 *                 progress kept in checkpoints (section 4.3)
 *   edl_shutdown  shutdown() (section 3.2)
 *
 * Conventions
 *   - every call returns 0 on success or a negative EDL_E* code;
 *     edl_last_error() gives a thread-local message for the last failure.
 *   - "dev" pointers are device memory owned by the caller; "host" pointers
 *     are ordinary host memory owned by the caller.  The library allocates no
 *     device memory.  A handle owns (until edl_shutdown) a few small pinned
 *     host staging buffers (the mini-batch's indices, the workers' losses),
 *     HIP events, and - unless the caller brings them, see
 *     edl_set_side_streams - two non-blocking streams of default priority.
 *   - device work is queued on the hipStream_t given to edl_init (NULL = the
 *     default stream).  A training pass also uses the two side streams (weight
 *     gradients; the update of layers whose gradients are final), ordered
 *     against the job's stream by events and joined to it before the call
 *     returns, so work queued on the job's stream afterwards sees the finished
 *     call.  Calls on one handle are not thread-safe.
 *   - launch heuristics and code-path switches live in one table of named
 *     integer options (edl_set_option / edl_get_option), each preset from
 *     the environment variable EDL_TUNE_<NAME> when the library is first used.
 *     They choose between paths that compute the same thing; none is needed
 *     for normal use.
 *   - tensors are channels-last: images [N][H][W][C], convolution weights
 *     [K][R][S][C]; parameters, momentum and gradients are float32 in one
 *     flat vector whose order is the model's layer order (see
 *     edl_tensor_info).
 */
#ifndef EDL_H
#define EDL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { EDL_OK = 0, EDL_EINVAL = -1, EDL_EINDIVISIBLE = -2, EDL_ENOMEM = -3, EDL_ERANGE = -4, EDL_EHIP = -5 };

/* The networks of the paper's evaluation (section 6) are all reachable: ResNet-50 / -101 / -152 are
 * EDL_MODEL_RESNET50 with stage depths {3,4,6,3} / {3,4,23,3} / {3,8,36,3}; VGG-16 / VGG-19 are
 * EDL_MODEL_VGG16 with group depths {2,2,3,3,3} / {2,2,4,4,4}; AlexNet is EDL_MODEL_ALEXNET. */
enum { EDL_MODEL_MLP = 0, EDL_MODEL_RESNET20 = 1, EDL_MODEL_RESNET50 = 2, EDL_MODEL_VGG16 = 3, EDL_MODEL_ALEXNET = 4 };

/* The variant of SGD that applies the aggregated gradient (section 2.1 names SGD "or its variants such
 * as Adam"; the usage example of section 3.2 wraps an Adam optimizer).  With g = aggregate + wd*w:
 *   MOMENTUM  v = momentum*v + g;  w -= lr*v
 *   ADAM      m = beta1*m + (1-beta1)*g;  s = beta2*s + (1-beta2)*g*g;
 *             w -= lr * (m / (1-beta1^t)) / (sqrt(s / (1-beta2^t)) + eps),   t = updates so far + 1
 *             (Algorithm 1 of Kingma & Ba; beta1 is the configuration's `momentum`). */
enum { EDL_OPT_MOMENTUM = 0, EDL_OPT_ADAM = 1 };

/* arithmetic type of activations and of the weight copies the matrix cores
 * read; master weights, momentum and gradients are float32 in both cases */
enum { EDL_DTYPE_F32 = 0, EDL_DTYPE_BF16 = 1 };

#define EDL_SNAPSHOT_MAGIC 0x314C4445u /* "EDL1" */
#define EDL_SNAPSHOT_HEADER_BYTES 256

typedef struct edl_handle edl_handle;

typedef struct edl_config {
    int32_t model;      /* EDL_MODEL_* */
    int32_t dtype;      /* EDL_DTYPE_* */
    int64_t N;          /* samples in the data set; a multiple of B */
    int64_t B;          /* aggregate mini-batch size, constant under scaling (section 3.1) */
    int32_t p_max;      /* largest parallelism the job will see (number of gradient buffers) */
    int32_t max_shard;  /* largest per-worker batch, B / (smallest p) */
    float lr, momentum, wd;
    /* geometry; 0 selects the model's default.  H, W, C: input image; classes: labels.
     * arch[] per model -
     *   MLP      {hidden1, hidden2}                     default {256, 256}; input is H*W*C features
     *   RESNET20 {width of stage 1, stages, blocks}     default {16, 3, 3}
     *   RESNET50 {base width, blocks of stages 1..4}    default {64, 3, 4, 6, 3}; 0 blocks ends the net
     *   VGG16    {base width, fc width, convolutions of groups 1..5}
     *                                                   default {64, 4096, 2, 2, 3, 3, 3}
     *   ALEXNET  {base width, fc width}                 default {64, 4096}; the five convolutions are
     *                                                   base x {1, 3, 6, 4, 4} wide */
    int32_t H, W, C, classes;
    int32_t arch[8];
    int32_t optimizer;  /* EDL_OPT_*; `momentum` above is Adam's beta1 */
    float beta2, eps;   /* Adam only: 0 <= beta2 < 1, eps >= 0 (ignored by EDL_OPT_MOMENTUM) */
} edl_config;

/* byte sizes and offsets inside the caller's arena (all offsets 256-byte aligned).  w, v, the second moment, the
 * bf16 copy and the gradient buffers start on 4 KB boundaries of alternating parity (offset bit 12), which is
 * what the update kernel runs fastest on; that holds in memory if the arena itself starts on an 8 KB boundary
 * (any 256-byte-aligned arena is correct). */
typedef struct edl_sizes {
    int64_t P;              /* parameters */
    int64_t R;              /* running-statistics floats (per batch-norm layer: mean[C], var[C]) */
    int64_t params_off;     /* float32 w[P] */
    int64_t momentum_off;   /* float32 v[P]: the momentum, or Adam's first moment */
    int64_t running_off;    /* float32 [R] */
    int64_t grads_off;      /* float32 G[p_max][P_padded] */
    int64_t grad_stride;    /* floats between consecutive workers' gradient buffers */
    int64_t arena_bytes;    /* total the caller must provide to edl_init */
    int64_t snapshot_bytes; /* EDL_SNAPSHOT_HEADER_BYTES + 4*(2P + R), with Adam 4*(3P + R) */
    double flops_per_sample; /* multiply-add flops of forward + both backward contractions */
    int64_t second_off;     /* float32 s[P]: Adam's second moment; -1 with EDL_OPT_MOMENTUM */
    int64_t scratch_bytes;  /* the part of the arena that is the kernels' scratch (what edl_step_static_scratch
                               must fit into EDL_STATIC_SCRATCH_BYTES) */
    int64_t shadow_off;     /* bf16 copy of w[P] that the contractions read; -1 for float32 jobs */
} edl_sizes;

/* progress of the job: what notify_batch_end() counts */
typedef struct edl_progress {
    int64_t step, epoch, step_in_epoch;
} edl_progress;

const char* edl_last_error(void);

/* Sizes for a configuration.  Host only; no GPU needed. */
int32_t edl_query(const edl_config* cfg, edl_sizes* out);

/* Number of parameter tensors and their place in the flat vector.  Host only.
 * name_buf receives a NUL-terminated name such as "s2.b1.conv2.w". */
int32_t edl_tensor_count(const edl_config* cfg, int32_t* out_count);
int32_t edl_tensor_info(const edl_config* cfg, int32_t i, char* name_buf, size_t name_cap,
                        int64_t* out_offset, int64_t* out_size, int64_t* out_fan_in);

/* He initialisation from the seed, as edl_init produces it.  Host only:
 * out_params is host float32[P].  Weights ~ N(0, 2/fan_in), biases 0,
 * batch-norm scale 1 and shift 0. */
int32_t edl_init_params_host(const edl_config* cfg, uint64_t seed, float* out_params);

/* Shard assignment (sections 3.1, 4.3).  Pure function of its arguments, host
 * only.  The epoch's permutation of 0..N-1 depends on (seed, epoch) only;
 * mini-batch `step_in_epoch` is its B consecutive entries from
 * step_in_epoch*B; worker k gets out_idx[out_off[k] .. out_off[k+1]).
 * out_idx: host int64[B]; out_off: host int64[p+1].
 * EDL_EINDIVISIBLE if B % p or N % B; EDL_ERANGE if step_in_epoch >= N/B. */
int32_t edl_shard_host(uint64_t seed, int64_t N, int64_t B, int32_t p, int64_t epoch,
                       int64_t step_in_epoch, int64_t* out_idx, int64_t* out_off);

/* Dynamic data pipeline (section 4.3): the leader's bookkeeping when the data
 * set is cut into d partitions (meta-data only) that workers are given on
 * demand.  Host only.  Partition j covers samples [j*s, min((j+1)*s, N)),
 * s = ceil(N/d) (EDL_EINVAL if that leaves a partition empty or d > N); each
 * epoch draws a permutation of the partitions from (seed, epoch) with the
 * job's generator, so d = N with a fixed worker set gives edl_shard_host's
 * assignment.
 *
 * edl_pipeline_next_batch assembles the next global mini-batch of B samples
 * for the p workers named by worker_ids (host int64[p], distinct, in rank
 * order; the caller chooses the names).  Workers of the previous call that
 * are missing have left gracefully: the unread rest of their current
 * partition goes back to the leader (in their old rank order) and is handed
 * out again before any unassigned partition, first in first out.  New names
 * are joiners and hold nothing.  Each worker is given B/p samples, read front
 * to back from its current partition and then from the next piece the leader
 * hands out; what a worker cannot be given because the epoch is running out
 * is passed on to the workers after it (wrapping round once), so the batch
 * has B samples but such a tail batch may have unequal shards.  An epoch ends
 * when all N samples have been handed out; the next call starts the next one.
 * out_idx: host int64[B]; out_off: host int64[p+1]; worker k reads
 * out_idx[out_off[k] .. out_off[k+1]).  EDL_EINDIVISIBLE if B % p or N % B.
 *
 * edl_pipeline_save writes the leader's state (progress, handed-back pieces,
 * every worker's partition and offset; the permutation follows from seed and
 * epoch) as int64 words: EDL_ENOMEM if cap_words is too small, *out_words then
 * holds the count to bring.  edl_pipeline_load creates a pipeline from such an
 * image (EDL_EINVAL / EDL_ERANGE if it is not one).  The caller owns the
 * pipeline until edl_pipeline_destroy.  Calls on one pipeline are not
 * thread-safe. */
typedef struct edl_pipeline edl_pipeline;
int32_t edl_pipeline_create(uint64_t seed, int64_t N, int64_t d, edl_pipeline** out);
int32_t edl_pipeline_next_batch(edl_pipeline* pl, int64_t B, int32_t p, const int64_t* worker_ids, int64_t* out_idx,
                                int64_t* out_off);
int32_t edl_pipeline_progress(const edl_pipeline* pl, int64_t* out_epoch, int64_t* out_consumed);
int32_t edl_pipeline_save(const edl_pipeline* pl, int64_t* buf, size_t cap_words, size_t* out_words);
int32_t edl_pipeline_load(const int64_t* buf, size_t words, edl_pipeline** out);
int32_t edl_pipeline_destroy(edl_pipeline* pl);

/* Create a job.  dev_arena: device memory of at least edl_query().arena_bytes,
 * 256-byte aligned, owned by the caller and alive until edl_shutdown.
 * Initialises parameters from the seed (He), zeroes momentum, sets running
 * statistics to mean 0 / variance 1, progress to 0. */
int32_t edl_init(edl_handle** out, const edl_config* cfg, uint64_t seed, void* dev_arena,
                 size_t arena_bytes, void* hip_stream);

/* The two streams a training pass uses beside the job's own (see Conventions): the caller's, which must
 * differ from each other and from the job's stream, be of default priority and outlive the handle's use of
 * them; or NULL, NULL for none (everything then runs on the job's stream).  Replaces whatever the handle used
 * before (streams the library created itself are destroyed).  Synchronises the job's stream and the old side
 * streams.  Results do not depend on the choice, bit for bit. */
int32_t edl_set_side_streams(edl_handle* h, void* wgrad_stream, void* update_stream);

/* Named integer options of the library (process-wide; see Conventions).  EDL_EINVAL for an unknown name.  Names:
 * force_tile (-1, or 0..3 = every forward / input-gradient launch on 128x128, 128x64, 128x32, 64x64 tiles),
 * wgrad_stream (1: jobs created from now on make their own side streams; 0: they do not), wgrad_tail_main,
 * early_update (least weights of a layer whose update starts during the backward pass; 0 = never),
 * early_blocks, join_tile, fused_stats, held_stats, fused_mask, fused_mask_cut, fused_mask_join,
 * min128, min128_long, bk64_kred, xcd, order, splitk_tiles, splitk_target, wgrad_blocks, wgrad_long_blocks,
 * small_tail_from, small_tail_to (64x64 launches of that many workgroups run with two LDS stages, all resident at once),
 * wgrad_long_ks, wgrad_deep_max (weight gradients of at most this many workgroups keep a third tile in flight), upd_vpt, upd_wide, upd_nt, upd_blocks (shape and cache hints of the update kernel's memory
 * walk), branch_stream (projection shortcuts on the second side stream), transpose_stream, alias_shortcut
 * (a shortcut's gradient read from the block output's gradient instead of copied), bn_nt, bn_nt_bytes
 * (non-temporal loads in the batch-norm passes for tensors of at least that many bytes), spare0, spare1. */
int32_t edl_set_option(const char* name, int64_t value);
int32_t edl_get_option(const char* name, int64_t* out_value);

/* The data set the shards index into: dev_x float32 [N][H][W][C], dev_y int32 [N]
 * (device memory, caller-owned, must stay alive). */
int32_t edl_bind_dataset(edl_handle* h, const float* dev_x, const int32_t* dev_y, int64_t N);

/* edl_shard_host with the job's seed and N. */
int32_t edl_shard(const edl_handle* h, int64_t B, int32_t p, int64_t epoch, int64_t step_in_epoch,
                  int64_t* out_idx, int64_t* out_off);

/* One synchronous mini-batch at parallelism p (sections 2.1, 3.1): for each
 * worker k, forward and backward on its shard into gradient buffer k; then the
 * p buffers are averaged and the fused momentum-SGD update
 *   g = mean_k G_k + wd*w ;  v = momentum*v + g ;  w = w - lr*v
 * is applied.  idx/off (host, as produced by edl_shard) may be NULL: then the
 * library takes the equal shards of its own progress cursor.
 * A caller's own cut may have shards of unequal size (a tail mini-batch of
 * edl_pipeline_next_batch; the current mini-batch redone by the survivors of a
 * failure, section 4.2's approximate recovery): off runs from 0 to B, every
 * shard has at most max_shard samples, a shard may be empty (that worker then
 * computes nothing), B need not be a multiple of p.  The aggregate is then
 * sum_k (n_k/B) G_k, which keeps the step the mean of the per-sample gradients
 * of the mini-batch; equal shards take the plain mean above (bit-identical to
 * it).  The first worker that has samples keeps the running statistics.
 * out_loss (host, may be NULL) receives the mean loss over the mini-batch
 * (the mean of the workers' mean losses, weighted by n_k/B if unequal); asking
 * for it synchronises the stream, otherwise the call only queues work.
 * Some of that work (weight gradients, the update of the largest layers) is
 * queued on streams of the library's own; it is joined to the handle's stream
 * before the call returns, so whatever the caller queues on that stream next
 * sees the finished step.
 * EDL_EINVAL p<=0 or p>p_max; without idx/off: EDL_EINDIVISIBLE B%p, EDL_ENOMEM
 * B/p>max_shard; with them: EDL_ENOMEM a shard larger than max_shard, EDL_ERANGE
 * index outside [0,N) or offsets not monotone from 0 to B. */
int32_t edl_step(edl_handle* h, int32_t p, const int64_t* idx, const int64_t* off, float* out_loss);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc) and so may have no room in their arena plan for the kernels' scratch: edl_step with that scratch
 * (split-reduction partial tiles, column-sum partials, batch-norm coefficients, per-row losses) in a buffer of
 * EDL_STATIC_SCRATCH_BYTES that the library holds once per GPU for the life of the process, instead of in the
 * arena's scratch piece.  The call allocates nothing, neither device nor pinned memory nor through any library;
 * arguments, results and errors are edl_step's, bit for bit the same model.  EDL_ENOMEM if the job's kernels
 * need more scratch than the buffer holds (large models: use edl_step); EDL_EINVAL if another device is current
 * than the one the job was created on.  All jobs on one GPU share the buffer, which keeps the last call's
 * contents: calls of this entry point that overlap on one GPU (other threads, other streams) race; calls that
 * follow each other on one stream, or are separated by a synchronisation, do not.  Nothing in the buffer needs
 * clearing between calls. */
#define EDL_STATIC_SCRATCH_BYTES (64u << 20)
int32_t edl_step_static_scratch(edl_handle* h, int32_t p, const int64_t* idx, const int64_t* off, float* out_loss);

/* Only the first half of edl_step (gradients of the p shards, no update).  For
 * parity tests and profiling. */
int32_t edl_gradients(edl_handle* h, int32_t p, const int64_t* idx, const int64_t* off, float* out_loss);

/* Only the second half: aggregate the gradient buffers of the last edl_gradients (by the mean, or by the
 * shards' shares if they were unequal) and update.  p must be that call's p.  The buffers are applied once:
 * EDL_EINVAL without a preceding edl_gradients, or on a second call after one. */
int32_t edl_apply(edl_handle* h, int32_t p);

/* The scheduler's profile(min_p, max_p) operator (sections 3.2, 5): the job is
 * run at every parallelism p in [min_p, max_p] that its configuration allows
 * (p divides B, p <= p_max, B/p <= max_shard), from the largest down to the
 * smallest, `steps` mini-batches each.  These are ordinary training steps: the
 * model and the progress move on exactly as by `steps` calls of edl_step per p.
 * Reported per p, timed with HIP events on the job's stream:
 *   ms_per_step, samples_per_s    one mini-batch of B samples on this GPU (all
 *                                 p shards back to back, then the update);
 *   worker_samples_per_s  t(p)    what one worker sustains on its shard of B/p
 *                                 samples: B / (time of the p gradient passes);
 *   efficiency            t(p) / max over the profiled p of t(p) (the paper's
 *                         GPU efficiency, with one GPU standing in for each
 *                         worker and no gradient exchange).
 * out: host array of cap entries, filled in the order run; *out_count = how
 * many.  EDL_EINVAL if no p in the range is allowed, steps <= 0 or steps > 256;
 * EDL_ENOMEM if cap is too small. */
typedef struct {
    int32_t p, shard;
    double ms_per_step, samples_per_s, worker_samples_per_s, efficiency;
} edl_parallelism_point;
int32_t edl_profile_parallelism(edl_handle* h, int32_t min_p, int32_t max_p, int32_t steps, edl_parallelism_point* out,
                                int32_t cap, int32_t* out_count);

/* State image for a joining worker: header, w[P], v[P], with Adam s[P], then
 * running[R] (float32, little endian), written to device memory dev_dst of
 * capacity cap.  The header carries the job's meta-data (section 4.2): model,
 * dtype, seed, N, B, progress, optimizer and its coefficients (lr, momentum,
 * wd; beta2, eps).  edl_restore refuses (EDL_EINVAL) an image of another model,
 * job size, optimizer or dtype (the worker's buffers were laid out for its
 * own), and ADOPTS the rest: seed, progress and the optimizer's coefficients
 * replace what the worker was created with, so a joiner continues exactly as
 * the job it joined.  Gradients pending from before the restore are void. */
int32_t edl_snapshot(edl_handle* h, void* dev_dst, size_t cap, size_t* out_written);
int32_t edl_restore(edl_handle* h, const void* dev_src, size_t len);

int32_t edl_get_progress(const edl_handle* h, edl_progress* out);

/* Test hooks: copy state to host float32 buffers (synchronise the stream). */
int32_t edl_get_params(edl_handle* h, float* host_dst /* [P] */);
int32_t edl_get_momentum(edl_handle* h, float* host_dst /* [P] */);
int32_t edl_get_running(edl_handle* h, float* host_dst /* [R] */);
int32_t edl_get_grad(edl_handle* h, int32_t k, float* host_dst /* [P] */);
int32_t edl_get_losses(edl_handle* h, int32_t p, float* host_dst /* [p] */);
int32_t edl_set_params(edl_handle* h, const float* host_src /* [P] */);
int32_t edl_set_momentum(edl_handle* h, const float* host_src /* [P] */);
/* Adam's second moment; EDL_EINVAL for a job with another optimizer */
int32_t edl_get_second_moment(edl_handle* h, float* host_dst /* [P] */);
int32_t edl_set_second_moment(edl_handle* h, const float* host_src /* [P] */);

/* Debugging hooks: run the two halves of one worker's pass separately and read
 * or overwrite activation tensors in between, so that a test can take the
 * sign / arg-max decisions of the backward pass from given activations.
 * Tensor 0 is the input batch; tensors are numbered in the order the layer
 * list creates them (a flattened view is a tensor of its own whose alias_of
 * names the tensor it shares storage with, else -1).  Host buffers are
 * float32 [n][H][W][C] whatever the job's dtype; `which` = 0 activation,
 * 1 gradient w.r.t. the activation.  All of these synchronise the stream.
 * edl_debug_set_tensor overwrites an activation (which = 0) or gradient (1) buffer.
 * edl_debug_forward: gather idx[0..n) (host) and run the forward pass, mean
 * loss readable through edl_get_losses(.., 1, ..); running statistics are not
 * touched.  edl_debug_backward: recompute the loss gradient from the current
 * logits and run the backward pass into gradient buffer k. */
int32_t edl_debug_tensor_count(const edl_handle* h, int32_t* out_count);
int32_t edl_debug_tensor_shape(const edl_handle* h, int32_t t, int32_t* H, int32_t* W, int32_t* C, int32_t* alias_of);
int32_t edl_debug_forward(edl_handle* h, const int64_t* idx, int32_t n);
int32_t edl_debug_backward(edl_handle* h, int32_t n, int32_t k);
int32_t edl_debug_get_tensor(edl_handle* h, int32_t t, int32_t which, int32_t n, float* host_dst);
int32_t edl_debug_set_tensor(edl_handle* h, int32_t t, int32_t which, int32_t n, const float* host_src);
/* One layer alone, on whatever its input buffers hold: forward writes the layer's
 * output activation (and the batch statistics / arg-max it keeps for its
 * backward); backward reads the gradient buffer of its output and overwrites
 * the gradient buffers of its inputs and its slice of gradient buffer k.  The
 * loss layer reads the labels given by edl_debug_set_labels (host int32[n]). */
int32_t edl_debug_op_count(const edl_handle* h, int32_t* out_count);
int32_t edl_debug_forward_op(edl_handle* h, int32_t op, int32_t n);
/* Layers op_lo .. op_hi-1 in order, as they run inside a step (a convolution
 * directly followed by its batch norm hands the batch statistics over instead
 * of the batch norm reading the tensor again). */
int32_t edl_debug_forward_range(edl_handle* h, int32_t op_lo, int32_t op_hi, int32_t n);
int32_t edl_debug_backward_op(edl_handle* h, int32_t op, int32_t n, int32_t k);
/* Layers op_hi-1 .. op_lo backward in that order, as they run inside a step (a
 * convolution's input-gradient pass can hand the masked gradient and its
 * column sums to the layer before it). */
int32_t edl_debug_backward_range(edl_handle* h, int32_t op_lo, int32_t op_hi, int32_t n, int32_t k);
/* The same when other readers of some tensors lie outside the range: the gradient buffers of the tensors in
 * held[0..n_held) already hold those readers' contribution (written with edl_debug_set_tensor) and the range
 * adds to it, as the readers inside a step find it at a residual join. */
int32_t edl_debug_backward_range_from(edl_handle* h, int32_t op_lo, int32_t op_hi, int32_t n, int32_t k,
                                      const int32_t* held, int32_t n_held);
int32_t edl_debug_set_labels(edl_handle* h, const int32_t* labels, int32_t n);

int32_t edl_shutdown(edl_handle* h);

/* Stand-alone aggregation + update on caller buffers (the aggregation step without a
 * model): dev_grads is a HOST array of p device pointers to float32[P];
 * dev_w, dev_v float32[P]; dev_w16 (may be NULL) receives the bf16 copy of the
 * updated weights, rounded to nearest even.  P need not be a multiple of
 * anything; pointers must be 16-byte aligned.  Any placement gives the same
 * bits; the kernel is fastest when the arrays start on 4 KB boundaries and
 * consecutive ones (dev_w / dev_v above all) differ in address bit 12, which
 * is how edl_query lays the same arrays out in a job's arena. */
int32_t edl_average_update(int32_t p, const float* const* dev_grads, float* dev_w, float* dev_v,
                           uint16_t* dev_w16, int64_t P, float lr, float momentum, float wd,
                           void* hip_stream);

/* The same with the Adam update (see EDL_OPT_ADAM): dev_m, dev_s float32[P] are the two moments, t >= 1
 * the number of this update (bias corrections 1/(1-beta^t) are formed on the host in double).  shares, if
 * not NULL, is a HOST array of p weights and the aggregate is sum_k shares[k]*G_k instead of the mean. */
int32_t edl_adam_update(int32_t p, const float* const* dev_grads, const float* shares, float* dev_w, float* dev_m,
                        float* dev_s, uint16_t* dev_w16, int64_t P, float lr, float beta1, float beta2, float eps,
                        float wd, int64_t t, void* hip_stream);

/* Measurement: with profiling on, every kernel launch of this library (any
 * handle, and the stand-alone calls) is bracketed by a HIP event pair on the
 * stream it is launched on.  edl_profile_report waits for those events, writes
 * a NUL-terminated JSON array of {"name","launches","ms","flops","bytes"}
 * (totals per kernel family; flops and bytes are the algorithmic work of the
 * launches) into buf and forgets the records.  EDL_ENOMEM if cap is too small
 * (out_needed then holds the size to bring). */
int32_t edl_profile(int32_t enable);
int32_t edl_profile_report(char* buf, size_t cap, size_t* out_needed);

/* Stand-alone vectorised device-to-device copy used by edl_snapshot. */
int32_t edl_copy(void* dev_dst, const void* dev_src, size_t bytes, void* hip_stream);

/* Measurement aid: a register-resident MFMA loop (no memory traffic), `blocks`
 * workgroups of four waves, `iters` rounds of four independent 32x32 MFMAs per
 * wave, in dtype's matrix instruction.  dev_sink: one float of device memory
 * (never written in practice).  out_flops receives the flops the launch issues;
 * time it with edl_profile ("mfma_rate_bf16" / "mfma_rate_f32").  What the
 * convolutions' MFMA fractions can be held against besides the data-sheet peak. */
int32_t edl_mfma_rate(int32_t dtype, int32_t blocks, int32_t iters, float* dev_sink, void* hip_stream, double* out_flops);

#ifdef __cplusplus
}
#endif
#endif /* EDL_H */
