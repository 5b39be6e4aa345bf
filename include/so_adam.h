/*
 * so_adam.h -- C ABI of the MI355X (gfx950) mixed-precision Adam(W) bucket-step library.
 *
 * The library implements, on one GPU, the optimizer hot path of the SuperOffload paper:
 * the per-bucket Adam step with its mixed-precision cast (Sec. 4.3, 4.5, 4.6), the global
 * gradient-norm / NaN-Inf validation (Sec. 4.4) and the speculative step with commit or
 * rollback (Sec. 4.4, speculation-then-validation), plus a host<->device bucket streamer
 * for optimizer state that lives in host memory (Sec. 4.3, the move/step/move pipeline).
 *
 * General conventions
 *   - Plain C types only.  "device" pointers are HIP device addresses owned by the caller;
 *     "host" pointers are ordinary host addresses.  The library never frees or reallocates
 *     caller memory.
 *   - All device arrays must be 16-byte aligned; element counts are arbitrary (tails are
 *     handled inside the kernels).
 *   - Every call enqueues its GPU work on the context's stream and returns without waiting,
 *     except the calls that fill a host `so_stats` (they synchronise that stream once) and
 *     so_stream_step / so_hybrid_step (they return after the whole pass has finished).
 *   - Errors are return codes; so_last_error(ctx) gives a message.  On an argument error no
 *     GPU work is enqueued and no caller state is modified.
 *   - Measurement and testing aids (event timing of the step kernels, lowered launch limits)
 *     are declared in so_adam_aux.h; they are not part of the method's boundary.
 *   - One context is used by one host thread at a time.
 */
#ifndef SO_ADAM_H
#define SO_ADAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct so_ctx so_ctx;

typedef enum so_status {
    SO_OK = 0,
    SO_ERR_INVALID_ARG = -1,   /* null pointer, n == 0 where not allowed, bad enum, step < 1 */
    SO_ERR_ALIGNMENT = -2,     /* a device pointer is not 16-byte aligned                    */
    SO_ERR_STATE = -3,         /* e.g. commit/rollback with nothing pending, double speculation */
    SO_ERR_OOM = -4,           /* a library-side allocation failed                           */
    SO_ERR_HIP = -5,           /* a HIP runtime call failed; message in so_last_error        */
    SO_ERR_UNSUPPORTED = -6
} so_status;

/* Gradient container types: 16-bit, as produced by a mixed-precision backward pass
 * (Sec. 4.5). */
enum { SO_GRAD_BF16 = 0, SO_GRAD_FP16 = 1 };

/* Type of the 16-bit working copy of the parameters (Sec. 4.5 speaks of FP16 throughout;
 * bf16 is the default of this build).  Both are round-to-nearest-even of the fp32 value. */
enum { SO_LP_BF16 = 0, SO_LP_FP16 = 1 };

/* Speculation modes of so_adam_step (Sec. 4.4, "in-place rollback"). */
enum {
    SO_SYNC = 0,          /* ordinary step: updates the current state in place               */
    SO_SPEC_PINGPONG = 1, /* reads the current set, writes the alt set; no extra traffic     */
    SO_SPEC_SAVE = 2      /* updates in place and writes the old p, m, v to the alt set;
                             40 B/param; rollback copies them back and re-derives the bf16
                             copy from the restored parameters                              */
};

/*
 * One flat bucket (Sec. 4.3: gradients, parameters and optimizer states are grouped into
 * fixed-size buckets).  Five parallel arrays of n elements; the same offset names the same
 * element in each.
 *
 *   grad        device, n 16-bit gradients (grad_dtype), read only
 *   param, exp_avg, exp_avg_sq   device, fp32 master parameter and Adam moments (current set)
 *   param_lp    device, n 16-bit working copy of param (lp_dtype), written by every step
 *   alt_*       device, a second set of the same four arrays; needed only for speculative
 *               steps, otherwise NULL.  alt_param_lp is not used in SO_SPEC_SAVE mode (the
 *               working copy is re-derived from the restored fp32 parameters).
 *   pending     managed by the library: 0, or the speculation mode of the uncommitted step.
 *
 * so_adam_commit in ping-pong mode SWAPS the current and alt pointers inside this struct;
 * the caller re-reads them afterwards.
 */
typedef struct so_bucket {
    const void* grad;
    float* param;
    float* exp_avg;
    float* exp_avg_sq;
    void* param_lp;
    float* alt_param;
    float* alt_exp_avg;
    float* alt_exp_avg_sq;
    void* alt_param_lp;
    uint64_t n;
    int32_t grad_dtype;
    int32_t pending;
    int32_t lp_dtype;        /* SO_LP_BF16 (0) or SO_LP_FP16 */
    int32_t reserved;
} so_bucket;

/* Adam hyper-parameters (the paper cites Adam and AdamW for its optimizer, Sec. 2.2; it
 * states no values).  adamw = 1: decoupled weight decay; 0: L2 decay added to the gradient.
 * bias_correction = 0 replaces 1 - beta^t by 1. */
typedef struct so_hparams {
    float lr;
    float beta1;
    float beta2;
    float eps;
    float weight_decay;
    int32_t adamw;
    int32_t bias_correction;
} so_hparams;

/* Global validation quantities (Sec. 4.4): sum of squares and L2 norm of the unscaled
 * gradients over finite elements, number of NaN/Inf gradient elements, and overflow =
 * (nonfinite > 0).  sumsq and norm are meaningful only when overflow == 0. */
typedef struct so_stats {
    double sumsq;
    double norm;
    uint64_t nonfinite;
    int32_t overflow;
    int32_t reserved;
} so_stats;

/* Outcome of validating one iteration (Sec. 4.4, the two rollback scenarios). */
enum { SO_COMMIT = 0, SO_ROLLBACK_SKIP = 1, SO_ROLLBACK_REDO = 2 };
typedef struct so_decision {
    int32_t action;          /* SO_COMMIT, SO_ROLLBACK_SKIP (NaN/Inf) or SO_ROLLBACK_REDO (clip) */
    int32_t reserved;
    double clip;             /* min(1, max_norm / (norm + 1e-6)); 1 when max_norm <= 0        */
    float grad_scale;        /* (float)(clip / loss_scale): the clip_coef to step with        */
    float next_loss_scale;   /* loss_scale, or max(loss_scale / 2, min_loss_scale) on overflow */
} so_decision;

/* One slice of a tensor inside a bucket, produced by so_layout_plan. */
typedef struct so_slice {
    uint64_t tensor;         /* index into the tensor list                                   */
    uint64_t tensor_offset;  /* first element of the slice inside the tensor                 */
    uint64_t bucket;         /* bucket index                                                 */
    uint64_t bucket_offset;  /* first element of the slice inside the bucket                 */
    uint64_t len;            /* elements                                                     */
} so_slice;

/* Timing report of so_stream_step. */
typedef struct so_stream_report {
    double total_ms;         /* wall time of the pass (work queued earlier is waited for first) */
    double h2d_gbps;         /* host->device bytes / busy time of the upload stream           */
    double d2h_gbps;         /* device->host bytes / busy time of the download stream         */
    double kernel_ms;        /* sum of the step kernels' durations                            */
    uint64_t buckets;
} so_stream_report;

/* Optimizer state that lives in pinned host memory (so_stream_step). */
typedef struct so_stream_state {
    float* host_param;       /* pinned host, n_total fp32                                     */
    float* host_exp_avg;     /* pinned host, n_total fp32                                     */
    float* host_exp_avg_sq;  /* pinned host, n_total fp32                                     */
    const void* grad;        /* device, n_total 16-bit gradients                              */
    void* param_lp;          /* device, n_total bf16 working copy (written)                   */
    uint64_t n_total;
    uint64_t bucket_elems;   /* elements per staged bucket (last one may be shorter)          */
    int32_t grad_dtype;
    int32_t lp_dtype;        /* SO_LP_BF16 (0) or SO_LP_FP16                                   */
    void* staging;           /* optional device workspace for the three staging slots (16-byte
                                aligned, caller-owned); NULL: the context allocates its own     */
    uint64_t staging_bytes;  /* size of `staging`: at least 36 * min(bucket_elems, n_total
                                rounded up to 8) bytes                                         */
} so_stream_state;

/* ---------------------------------------------------------------------------------------
 * Context
 * ------------------------------------------------------------------------------------- */

/* Library version string (static storage). */
const char* so_version(void);

/* Create a context on HIP device `device`.  `hip_stream` is a hipStream_t (NULL = the
 * default stream) on which all work of this context is enqueued.  The context owns about
 * 65 MiB of device scratch (reduction partials, bucket tables) and a pinned result slot;
 * the streaming calls add three staging slots on first use. */
so_status so_create(so_ctx** out, int device, void* hip_stream);

/* Waits for the context's stream, frees everything the context owns.  NULL is allowed. */
so_status so_destroy(so_ctx* ctx);

/* Switch the stream used by later calls.  Work already enqueued stays on the old stream; the
 * caller orders the two streams (an event or a synchronisation) wherever later calls depend
 * on earlier ones -- in particular between so_grad_stats_enqueue and so_adam_step_guarded, and
 * between speculative steps and so_adam_step_stats. */
so_status so_set_stream(so_ctx* ctx, void* hip_stream);

/* Message of the last failed call on this context ("" if none).  Valid until the next call.
 * ctx == NULL: message of the last failed so_grad_stats_static call on the calling thread. */
const char* so_last_error(const so_ctx* ctx);

/* ---------------------------------------------------------------------------------------
 * Bucket layout (Sec. 4.3: bucketisation).  Host-only integer work.
 * ------------------------------------------------------------------------------------- */

/* Flatten `nt` tensors (element counts in tensor_numel, model order) back to back and cut
 * the flat index space every `bucket_elems` elements.  Writes the slices in flat order to
 * out[0..cap) and the number of slices / buckets to *n_slices / *n_buckets.  With out ==
 * NULL only the counts are computed.  SO_ERR_INVALID_ARG if cap is too small. */
so_status so_layout_plan(const uint64_t* tensor_numel, size_t nt, uint64_t bucket_elems,
                         so_slice* out, size_t cap, size_t* n_slices, uint64_t* n_buckets);

/* Where to put the five flat arenas of a model (all buckets of one array kind back to back,
 * n_total elements each) inside ONE device allocation -- the data layout in HBM this library is
 * measured with.  Order p, g, m, q, v: the 16-bit arrays lie between the fp32 arrays, so the
 * three fp32 streams that a step reads and writes at the same index lie 1.5 array lengths
 * apart.  In physically contiguous memory (an allocation made at start-up on an otherwise
 * empty device) the step over the 8-billion-parameter workload runs 2 % faster in this
 * order than with the arrays in the order p, m, v, g, q or in five separate allocations;
 * it was never measured slower.  All offsets are multiples of 2 MiB and are relative to a
 * base the caller aligns to 2 MiB (or at least 16 bytes); `bytes` is the size to allocate,
 * including 2 MiB of slack for that alignment.  Pure host arithmetic.  Buckets are then
 * index ranges of the arenas: bucket k's arrays start at element k * bucket_elems of each. */
typedef struct so_arena_layout {
    uint64_t bytes;          /* size of the allocation                                        */
    uint64_t param;          /* byte offset of the fp32 parameters (n_total * 4 bytes)        */
    uint64_t grad;           /* ... of the 16-bit gradients (n_total * 2 bytes)               */
    uint64_t exp_avg;        /* ... of the fp32 first moments                                 */
    uint64_t param_lp;       /* ... of the 16-bit working copy                                */
    uint64_t exp_avg_sq;     /* ... of the fp32 second moments                                */
} so_arena_layout;
so_status so_arena_plan(uint64_t n_total, so_arena_layout* out);

/* Placement by measurement.  How fast the step streams its arrays depends on where they lie
 * in the device's physical memory relative to each other (at the scale of gigabytes; +-2.5 %
 * for the in-place step and +-4 % for the ping-pong step on MI355X), and a process cannot see
 * physical addresses -- but it can time the step.  Given a device workspace LARGER than the
 * state (workspace_bytes; the more slack, the more placements there are to choose from),
 * so_arena_tune times the step kernel itself on candidate placements of the arenas inside it:
 * first the tight so_arena_plan layout at the workspace's start, then `trials` random orders,
 * every other one with random gaps (a workspace of exactly the state's size leaves only the
 * order to choose; drawn from a generator seeded with `seed`: same seed, same candidates), then moves
 * of single arenas around the best one found; the four fastest and the tight layout are then
 * timed once more, four steps each, and the fastest by that comparison is returned in *out
 * (offsets relative to `workspace`, which needs no alignment: arenas start at multiples of
 * 2 MiB from its first 16-byte boundary; out->bytes = end of the last arena).  The result is
 * never slower, by the call's own measurement, than the tight layout.
 *   out_alt == NULL   the five arenas of the in-place step are placed;
 *   out_alt != NULL   the four arenas of a second state set (ping-pong speculation) are placed
 *                     as well, and the ping-pong step is timed in both directions.
 *   trials == 0       the tight layout is returned without timing anything.
 *   tight_ms, tuned_ms (optional, host) receive the step-kernel time of the tight and of the
 *                     returned placement, in milliseconds per step.
 * The CONTENTS of the workspace are overwritten (filled with a finite pattern, then stepped):
 * call this at set-up, before the state is initialised; the arenas hold arbitrary values
 * afterwards.  Takes at most (trials + 18 x arenas + 20) x 3 steps of the whole state
 * on the context's stream and returns when done; must not be recorded into a graph.
 * SO_ERR_INVALID_ARG if the workspace cannot hold the arenas, n_total is 0 or trials > 4096;
 * SO_ERR_STATE if statistics of speculative steps are pending in the context. */
typedef struct so_arena_alt {
    uint64_t param, exp_avg, exp_avg_sq, param_lp;      /* byte offsets of the second state set */
} so_arena_alt;
/* The candidates of so_arena_tune's search, as pure host arithmetic: the index-th placement of
 * the arenas of n_total parameters inside a workspace of workspace_bytes whose base is 16-byte
 * aligned.  index 0 is the tight so_arena_plan layout (second set, if asked for, behind it in
 * the order p' m' v' q'); every index > 0 is a random order of the arenas drawn from (seed,
 * index) alone -- packed tightly if index is odd or the workspace has no room to spare, with
 * random gaps (multiples of 1/256 of the spare room, rounded down to 2 MiB) otherwise.  Every
 * arena starts at a multiple of 2 MiB and no two overlap; out->bytes is the end of the last
 * one and never exceeds workspace_bytes.  out_alt == NULL: five arenas.  SO_ERR_INVALID_ARG if
 * the workspace cannot hold the arenas or n_total is 0 or too large for so_arena_plan. */
so_status so_arena_candidate(uint64_t n_total, uint64_t workspace_bytes, uint64_t seed, uint32_t index,
                             so_arena_layout* out, so_arena_alt* out_alt);
so_status so_arena_tune(so_ctx* ctx, void* workspace, uint64_t workspace_bytes, uint64_t n_total,
                        int grad_dtype, uint32_t trials, uint64_t seed, so_arena_layout* out,
                        so_arena_alt* out_alt, double* tight_ms, double* tuned_ms);

/* Gather tensor slices into flat bucket arrays (or scatter them back) on the GPU.
 * tensors[i] is the device address of tensor i, buckets[k] the device address of bucket
 * k's flat array, both holding elements of elem_size bytes (2 or 4).  Addresses must be
 * multiples of the element size (SO_ERR_ALIGNMENT otherwise); nothing more is required, but
 * a slice whose source and destination sit at the same offset inside their 16-byte granules
 * (always the case for 16-byte-aligned bases and tensor sizes that are multiples of 8
 * elements) copies about 15 % faster than one that does not.
 * direction 0: tensors -> buckets, 1: buckets -> tensors.  The copy is enqueued on the
 * context's stream like every other call; the slice table is kept in context-owned memory
 * (grown on demand: a call with more slices than any before allocates), so `slices`,
 * `tensors` and `buckets` (the host arrays) may be reused on return. */
so_status so_flatten(so_ctx* ctx, const so_slice* slices, size_t n_slices,
                     void* const* tensors, void* const* buckets, int elem_size, int direction);

/* Gather 16-bit gradient tensors into their buckets (so_flatten with elem_size 2, direction 0)
 * and obtain the validation quantities of Sec. 4.4 from the same pass: every gradient is read
 * once, copied, and entered into the sum of squares and the NaN/Inf count.  The result is left
 * on the GPU exactly as so_grad_stats_enqueue over the filled buckets would leave it (same
 * meaning of loss_scale and max_norm; statistics cover the elements the slices name), so
 * so_adam_step_guarded or so_grad_stats_fetch may follow.  Saves the separate 2-byte-per-element
 * statistics pass whenever gradients arrive as per-tensor arrays.  grad_dtype: SO_GRAD_BF16 or
 * SO_GRAD_FP16.  SO_ERR_STATE if speculative steps have left the partial buffer (4 Mi entries)
 * too full; fetch their statistics first. */
so_status so_flatten_grad_stats(so_ctx* ctx, const so_slice* slices, size_t n_slices,
                                void* const* tensors, void* const* buckets, int grad_dtype,
                                float loss_scale, float max_norm);

/* ---------------------------------------------------------------------------------------
 * Validation quantities (Sec. 4.4)
 * ------------------------------------------------------------------------------------- */

/* Global gradient statistics over buckets[0..nb): reads every bucket's grad once (2 bytes
 * per element), two-stage deterministic reduction, result copied to *out_host after one
 * stream synchronisation.  Gradients are multiplied by inv_loss_scale before squaring.
 * Only grad, n and grad_dtype of each bucket are used.  nb == 0 gives all zeros. */
so_status so_grad_stats(so_ctx* ctx, const so_bucket* buckets, size_t nb,
                        float inv_loss_scale, so_stats* out_host);

/* For callers that cannot allocate -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: the same global statistics as so_grad_stats, through an
 * entry point that needs no context and calls no hipMalloc, hipFree or other allocating
 * routine.  Its only scratch (the stage-1 partials, 64 KiB) is a static device array inside
 * the library, which every GPU the library runs on holds until the process ends; the bucket
 * list travels in the kernel arguments.
 *   buckets, nb     host array; only grad, n and grad_dtype of each bucket are used (grad:
 *                   device, 16-byte aligned, on the CURRENT HIP device).  At most
 *                   SO_STATIC_MAX_BUCKETS buckets with n > 0 per call: more is refused with
 *                   SO_ERR_UNSUPPORTED (split the list, or use so_grad_stats).  Element counts
 *                   are not limited.
 *   hip_stream      hipStream_t the two kernels are launched on (NULL = default stream)
 *   out_device      DEVICE memory, caller-owned, 8-byte aligned: receives one so_stats when the
 *                   stream reaches that point.  No synchronisation, no host copy.
 * Same grid, tile order and arithmetic as so_grad_stats, hence the same bits.  All calls on one
 * GPU share that GPU's scratch array: calls that overlap in time on one GPU (different
 * streams or threads) race; calls on one stream, or otherwise ordered, do not.  Nothing has to
 * be cleared between calls.  The device address of the array is looked up once per device
 * (by so_create, else by the first call on that device); a caller that captures a graph does
 * one of the two before the capture.  Errors: return code; message via so_last_error(NULL). */
#define SO_STATIC_MAX_BUCKETS 128
so_status so_grad_stats_static(const so_bucket* buckets, size_t nb, float inv_loss_scale,
                               void* hip_stream, so_stats* out_device);

/* Same reduction, but no synchronisation: the result stays in the context's device slot
 * for so_adam_step_guarded.  max_norm and loss_scale are used to derive, on the GPU, the
 * gradient multiplier clip / loss_scale and the skip flag. */
so_status so_grad_stats_enqueue(so_ctx* ctx, const so_bucket* buckets, size_t nb,
                                float loss_scale, float max_norm);

/* Host copy of the result of the last so_grad_stats_enqueue (synchronises the stream). */
so_status so_grad_stats_fetch(so_ctx* ctx, so_stats* out_host, so_decision* decision_host);

/* ---------------------------------------------------------------------------------------
 * Autonomous iterations: the validator of Sec. 4.4 entirely on the GPU
 * ------------------------------------------------------------------------------------- */

/* The synchronous iteration -- statistics, validation, guarded step -- with everything that
 * carries over from one iteration to the next kept in device memory: Adam's step count t
 * (advanced only when a step is applied), the bias-correction powers beta^t, the loss scale
 * (halved on NaN/Inf, doubled after growth_interval clean iterations in a row, 0 = never;
 * see so_loss_scale_next) and the clip coefficient min(1, max_norm / (norm + 1e-6)).  A
 * training loop therefore calls so_train_iteration once per iteration and never waits for the
 * GPU; so_train_fetch is for logging.
 *
 * so_train_reset   fixes hyper-parameters (one set for all buckets), the count of the first
 *                  step (1 for a fresh run), the loss-scale policy and max_norm (<= 0: no
 *                  clipping); synchronises the stream once.
 * so_train_iteration   enqueues three launches on the context's stream: statistics over all
 *                  buckets' gradients, the validation kernel, the fused step of all buckets
 *                  (skipped by the GPU itself on NaN/Inf).  Buckets as for so_adam_step_multi.
 * so_train_fetch   waits for the stream; statistics and decision of the last iteration,
 *                  number of steps applied so far, and the loss scale the next iteration will
 *                  use.  Any out pointer may be NULL.
 * The result equals the same sequence of so_grad_stats_enqueue / so_adam_step_guarded calls
 * driven from the host, up to the last bit of the bias-correction factors (running products
 * instead of pow). */
so_status so_train_reset(so_ctx* ctx, const so_hparams* hp, int64_t first_step, float loss_scale,
                         float min_loss_scale, float max_loss_scale, uint32_t growth_interval,
                         float max_norm);
so_status so_train_iteration(so_ctx* ctx, so_bucket* buckets, size_t nb);
so_status so_train_fetch(so_ctx* ctx, so_stats* out_host, so_decision* decision_host,
                         int64_t* applied_steps, float* loss_scale);

/* The launches of so_train_iteration over a fixed list of buckets recorded once as a HIP graph
 * and replayed with one call per iteration: for small optimizer states, where the iteration
 * is bound by launch overhead rather than by HBM.  Nothing that changes between iterations is
 * a launch argument (step count, loss scale and the step's scalars are read from device
 * memory), so the same graph serves every iteration.
 *   so_train_capture  records (no GPU work runs); the bucket pointers and sizes are frozen
 *                     into the graph -- the caller refills the same gradient arrays before
 *                     each replay.  Needs so_train_reset first; a new capture replaces the old.
 *   so_train_replay   launches the recorded iteration on the context's stream.
 * Replays and so_train_iteration calls may be mixed freely; both advance the same train state. */
so_status so_train_capture(so_ctx* ctx, so_bucket* buckets, size_t nb);
so_status so_train_replay(so_ctx* ctx);

/* Pure host function: turn statistics into the iteration's outcome.  In a speculative
 * schedule the step already ran with clip = 1: overflow -> SO_ROLLBACK_SKIP, clip < 1 ->
 * SO_ROLLBACK_REDO with grad_scale, else SO_COMMIT.  A synchronous schedule uses the same
 * fields: skip on overflow, otherwise step with grad_scale. */
so_status so_validate(const so_stats* stats, double max_norm, double loss_scale,
                      double min_loss_scale, so_decision* out);

/* Dynamic loss scaling around so_validate (Sec. 4.4 names the NaN/Inf check of mixed-precision
 * training; the schedule is not given by the paper, this is the usual one): on overflow the
 * scale is halved (not below min_loss_scale) and the count of clean iterations restarts;
 * otherwise the count goes up by one and, when it reaches growth_interval (0 = never grow),
 * the scale doubles (not above max_loss_scale) and the count restarts.  Pure host function;
 * *clean_iterations is caller-owned state, 0 at the start of training. */
so_status so_loss_scale_next(float loss_scale, int overflow, uint32_t* clean_iterations,
                             uint32_t growth_interval, float min_loss_scale,
                             float max_loss_scale, float* next_loss_scale);

/* ---------------------------------------------------------------------------------------
 * The fused Adam(W) + cast step (Sec. 4.6 GraceAdam, Sec. 4.5 casting)
 * ------------------------------------------------------------------------------------- */

/*
 * One step over one bucket.  Per element, in fp32:
 *     g' = g * clip_coef                      (+ weight_decay * p when adamw == 0)
 *     m  = beta1 m + (1 - beta1) g'
 *     v  = beta2 v + (1 - beta2) g'^2
 *     p  = p - lr wd p - (lr / (1 - beta1^step)) m / (sqrt(v) / sqrt(1 - beta2^step) + eps)
 *     param_lp = round_to_nearest_even_16bit(p)          (bf16, or fp16 if lp_dtype says so)
 * 28 bytes of memory traffic per element.  `step` is the 1-based count of applied steps.
 * clip_coef is the multiplier applied to every gradient (clip / loss_scale).
 *
 * speculative == SO_SYNC: in place.  SO_SPEC_PINGPONG / SO_SPEC_SAVE: see the enum; the
 * kernel additionally accumulates the gradient statistics of the bucket (sum of squares of
 * g * clip_coef over finite g, count of non-finite g) for so_adam_step_stats, and sets
 * b->pending.  A bucket with pending != 0 cannot be stepped again (SO_ERR_STATE).
 */
so_status so_adam_step(so_ctx* ctx, so_bucket* b, const so_hparams* hp, int64_t step,
                       float clip_coef, int speculative);

/* The same step over buckets[0..nb) in ONE kernel launch (buckets may have different n;
 * all must have the same grad_dtype). */
so_status so_adam_step_multi(so_ctx* ctx, so_bucket* buckets, size_t nb, const so_hparams* hp,
                             int64_t step, float clip_coef, int speculative);

/* The same single launch with one so_hparams PER BUCKET (parameter groups: e.g. no weight
 * decay or another learning rate for some buckets); hp_per_bucket has nb entries. */
so_status so_adam_step_groups(so_ctx* ctx, so_bucket* buckets, size_t nb,
                              const so_hparams* hp_per_bucket, int64_t step, float clip_coef,
                              int speculative);

/* Synchronous step whose gradient multiplier and skip flag are read ON THE GPU from the
 * result of so_grad_stats_enqueue: no host round trip between validation and step.  If the
 * statistics say overflow, the kernel leaves all state untouched. */
so_status so_adam_step_guarded(so_ctx* ctx, so_bucket* buckets, size_t nb,
                               const so_hparams* hp, int64_t step);

/* Statistics accumulated by the speculative steps issued since the last call of this
 * function (or since so_create): second reduction stage + one stream synchronisation.
 * This is the validation of Sec. 4.4 obtained as a by-product of the step itself. */
so_status so_adam_step_stats(so_ctx* ctx, so_stats* out_host);

/* Accept a speculative step.  Ping-pong: O(1), swaps current and alt pointers in *b.
 * Save mode: O(1), the saved copy is simply dropped.  SO_ERR_STATE if nothing is pending. */
so_status so_adam_commit(so_ctx* ctx, so_bucket* b);

/* Undo a speculative step bit for bit, including the bf16 working copy.  Ping-pong: O(1),
 * the alt set is dropped.  Save mode: copies the saved p, m, v back (28 bytes/param incl.
 * the working copy).  SO_ERR_STATE if nothing is pending. */
so_status so_adam_rollback(so_ctx* ctx, so_bucket* b);

/* ---------------------------------------------------------------------------------------
 * Streaming step for optimizer state in host memory (Sec. 4.3)
 * ------------------------------------------------------------------------------------- */

/* Bucket repartitioning (Sec. 4.3, the inequality that fixes how many of the last buckets
 * keep their optimizer state on the GPU): the smallest n <= min(n_buckets, max_resident) with
 *     move_grad + step_offloaded + move_param  <=  n * (bwd_per_bucket + step_resident_per_bucket)
 * i.e. the offloaded path of one bucket hides behind the backward pass and resident step of
 * n buckets; n = the cap if no n satisfies it.  Pure host arithmetic on measured times (ms). */
so_status so_plan_resident(double move_grad_ms, double step_offloaded_ms, double move_param_ms,
                           double bwd_ms_per_bucket, double step_resident_ms_per_bucket,
                           uint64_t n_buckets, uint64_t max_resident, uint64_t* n_resident);

/* Page-locked host memory for so_stream_step (Sec. 4.5: transfers through unpinned memory
 * are much slower).  Plain hipHostMalloc / hipHostFree; *out is a host pointer. */
so_status so_pinned_alloc(size_t bytes, void** out);
so_status so_pinned_free(void* ptr);

/* One synchronous-schedule step over state kept in pinned host memory: bucket k+1 is
 * uploaded and bucket k-1 downloaded on two side streams while bucket k is stepped in
 * device staging slots -- three slots of 12 * bucket_elems bytes, in the workspace
 * st->staging if the caller gives one, else owned by the context and allocated on first use.  Returns when the pass is complete.  Result is bit-identical to
 * stepping the same data resident on the device.
 * Error behaviour: argument errors are reported before anything is queued.  If a HIP call
 * fails in the middle of the pass, all streams the pass uses are drained before the call
 * returns SO_ERR_HIP; the host arrays may then be freed or reused, but their contents are
 * undefined (some buckets stepped, others not). */
so_status so_stream_step(so_ctx* ctx, const so_stream_state* st, const so_hparams* hp,
                         int64_t step, float clip_coef, so_stream_report* report);

/* The repartitioned step of Sec. 4.3: part of the optimizer state stays on the GPU (the last
 * buckets of the model) and the rest lives in host memory.  The `n_resident` device-resident
 * buckets take the ordinary synchronous step (as so_adam_step_multi, same hyper-parameters,
 * same step count and clip coefficient) on a side stream owned by the context, queued before
 * the first transfer, so that their kernels run while the host link moves the streamed
 * buckets of `st` (as so_stream_step).  Returns when both parts are complete; the main
 * stream resumes after both.  Results are bit-identical to the two separate calls.
 * `report` (optional) describes the streamed part; `resident_ms` (optional, host) receives the
 * time from the first resident kernel's start to the last one's end, which includes whatever
 * the concurrent streamed kernels and transfers cost it.  n_resident == 0 is so_stream_step;
 * st->n_total == 0 is so_adam_step_multi.  Errors in the resident buckets are reported before
 * anything is queued. */
so_status so_hybrid_step(so_ctx* ctx, const so_stream_state* st, so_bucket* resident,
                         size_t n_resident, const so_hparams* hp, int64_t step, float clip_coef,
                         so_stream_report* report, double* resident_ms);

/* ---------------------------------------------------------------------------------------
 * Working copy from fp32 parameters: the cast on the GPU side of the link (Sec. 4.5)
 * ------------------------------------------------------------------------------------- */

/* param_lp[i] = param[i] rounded to lp_dtype (SO_LP_BF16 / SO_LP_FP16, round to nearest even,
 * NaN stays NaN, overflow goes to infinity): exactly the rounding the step applies when it stores
 * the working copy, so the result equals what a step that stored the same parameters left
 * behind.  Both arrays in device memory, 16-byte aligned (SO_ERR_ALIGNMENT otherwise), n
 * elements; enqueued on the context's stream.  n == 0 is a no-op. */
so_status so_cast_params(so_ctx* ctx, const float* param, void* param_lp, uint64_t n, int lp_dtype);

/* The same with the fp32 parameters in HOST memory (pinned for full link rate, pageable
 * accepted): the transfer-then-cast form of Sec. 4.5 -- 4 bytes per parameter cross the host
 * link in chunks of chunk_elems (a positive multiple of 8) into the context's staging slots,
 * and each chunk is cast on the GPU while the next one is on its way.  param_lp: device, 16-byte
 * aligned, n elements.  Returns when the copy is complete; total_ms (optional, host) receives
 * the wall time of the pass, measured after the work queued earlier on the context's stream has
 * finished.  Staging slots are allocated on first use and grown on demand, as for
 * so_stream_step.  Errors as so_stream_step: arguments are checked before anything is queued,
 * and after a HIP failure in mid-pass the streams are drained before the call returns. */
so_status so_stream_cast_params(so_ctx* ctx, const float* host_param, void* param_lp, uint64_t n,
                                uint64_t chunk_elems, int lp_dtype, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* SO_ADAM_H */
