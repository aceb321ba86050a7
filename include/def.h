/*
 * def.h -- C ABI of the DEF / DEF-A compression-and-update step with random
 * block-wise gradient sparsification (RBGS) for one AMD MI355X (gfx950).
 *
 * Method: Xu & Huang, "Detached Error Feedback for Distributed SGD with Random
 * Sparsification" (arXiv 2004.05298).  One call of def_step / def_a_step is one
 * iteration t of Algorithm 1 for all W (the paper's K) data-parallel workers,
 * whose gradients, error memories and momentum buffers all live on this GPU:
 *
 *   m_k <- mu*m_k + g_k                       Sec. 3.2 "Momentum Variant", Eq. (11)
 *   p_k  = eta*m_k + e_k                      Algorithm 1, error-feedback line
 *   e_k <- p_k - C(p_k)                       Algorithm 1, residual line
 *   C(p) = (1/W) sum_k C(p_k)                 Algorithm 1, ring-allreduce line
 *   x   <- x - C(p)                           Algorithm 1, update line
 *
 * C is RBGS (Sec. 1): it keeps one contiguous block of the flattened vector and
 * zeroes the rest; every worker draws the same block from a shared seed.
 *
 * Conventions
 *   - All floating-point buffers are IEEE binary32; every multiply and add is
 *     rounded separately (no fused multiply-add), so results do not depend on
 *     the launch shape.
 *   - "DEVICE" pointers are HIP device memory on the GPU that was current when
 *     def_init was called (the stream must belong to it too); "HOST" pointers
 *     are ordinary process memory.  Later calls make that GPU current while
 *     they run and put the caller's back before they return, so a process that
 *     drives several GPUs need not switch devices around calls into a context.
 *   - Every function returns DEF_OK (0) or a negative def_status.  No function
 *     throws or aborts.  A call that returns DEF_EINVAL has changed nothing.
 *     A step that returns DEF_EHIP because its streaming launch (or anything before
 *     it) failed has not advanced the step counter, has consumed no forced start and
 *     has changed no state buffer; with the device draw on, the device's copy of the
 *     counter is put back to the host's on the same stream.  If a later launch of the
 *     same step fails (the separate averaging kernel, the y output) the streaming
 *     pass has already been enqueued: the context is then mid-step and must be
 *     destroyed or have its state restored from a checkpoint.
 *   - def_step / def_a_step / def_output only enqueue work on the context's
 *     stream and return; they never synchronise with the device.
 *   - A context is not thread-safe; use one context per host thread.
 */
#ifndef DEF_H_
#define DEF_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum def_status {
    DEF_OK = 0,
    DEF_EINVAL = -1,   /* bad argument: NULL pointer, bad shape, bad offset table, ld < d, ... */
    DEF_ENOMEM = -2,   /* device or host allocation failed                                      */
    DEF_EHIP = -3,     /* a HIP runtime call failed; def_last_hip_error() has its code          */
    DEF_ELIMIT = -4    /* the problem exceeds a fixed limit of the entry point called           */
} def_status;

typedef struct def_ctx def_ctx; /* opaque, owned by the library */

/*
 * Problem statement (Algorithm 1 "Input"; Sec. 3.2 for mu; Sec. 1 for the seed).
 */
typedef struct def_config {
    uint64_t d;             /* number of parameters, 1 <= d < 2^40                              */
    uint32_t W;             /* number of workers (the paper's K), >= 1; W * (ceil(d/256) + 7) must be
                               below 2^31 (one workgroup per worker and 256 indices)            */
    uint32_t R;             /* compression ratio, integer, 1 <= R <= d.  The kept block has
                               B = ceil(d/R) elements (delta = B/d, Assumption 4.2).            */
    float lr;               /* learning rate eta                                                */
    float momentum;         /* mu.  0 selects Algorithm 1 as printed: p = eta*g + e, and no
                               momentum buffer is allocated.                                    */
    float weight_decay;     /* wd.  0 = off.  Otherwise g' = g + wd*x_t replaces g (decay folded
                               into the gradient at the shared iterate, before momentum).       */
    uint64_t seed;          /* shared random seed of the block draw                             */
    const uint64_t *tensor_offsets; /* HOST, n_tensors+1 entries: off[0]=0 < off[1] < ... <
                               off[n_tensors]=d.  Tensor l of the model occupies flat indices
                               [off[l], off[l+1]).  NULL means one tensor of length d.  Copied. */
    uint32_t n_tensors;     /* L >= 1 (ignored when tensor_offsets is NULL)                     */
    float *params;          /* DEVICE, d floats: the model x as ONE flat vector, caller-owned,
                               updated in place.  NULL selects tensor mode (param_ptrs).        */
    float *const *param_ptrs; /* HOST array of n_tensors DEVICE pointers; tensor l has
                               off[l+1]-off[l] floats, caller-owned, updated in place.  Used
                               only when params == NULL.  The array is copied.                  */
    void *stream;           /* hipStream_t all work is enqueued on (NULL = the null stream)     */
} def_config;

/*
 * Create a context: validates cfg, allocates and zero-fills the W error
 * memories (e_{k,0}=0, Algorithm 1 "Initialize"), the W momentum buffers
 * (m_{k,0}=0, Sec. 3.2) unless momentum == 0, the compact message buffer
 * [W][B] and the averaged block [B].  Step counter t starts at 0.
 * *out is written only on success.  Synchronises the stream once.
 */
int def_init(def_ctx **out, const def_config *cfg);

/* Frees everything def_init allocated (synchronises the stream first). */
int def_destroy(def_ctx *ctx);

/*
 * One DEF iteration (Algorithm 1, inner loop, with the momentum variant).
 *   grads  DEVICE, read-only: worker k's flat gradient g_{k,t} starts at
 *          grads + k*ld; ld >= d elements.  Tensor l sits at +off[l].  Must stay
 *          valid until the stream has executed the step.  Any 4-byte alignment
 *          and any ld >= d are accepted; 16-byte aligned rows (ld a multiple of 4)
 *          are fast, rows that start on 1 KiB boundaries (grads 1 KiB-aligned and ld
 *          a multiple of 256) are fastest.
 *   y_out  DEVICE or NULL.  If not NULL, d floats receive DEF's output
 *          y_{t+1} = x_{t+1} - (1/W) sum_k e_{k,t+1}   (Algorithm 1 "Output";
 *          Sec. 3.2, Eq. (8)).  The paper needs y only when the model is
 *          evaluated, so pass NULL in the training loop.
 * Draws s_t = def_block_start(seed, t, d) (or the forced start), keeps the
 * circular block {(s_t + j) mod d : 0 <= j < B}, then t <- t+1.
 */
int def_step(def_ctx *ctx, const float *grads, uint64_t ld, float *y_out);

/*
 * One DEF-A iteration.  DEF-A runs the same iteration as DEF and returns x_T
 * instead of y_T (Algorithm 1 "Output"; Sec. 3.2 "DEF-A"), so this is def_step
 * with no y: after it, params holds DEF-A's model.
 */
int def_a_step(def_ctx *ctx, const float *grads, uint64_t ld);

/*
 * Tensor mode of the two steps: gradients are given per tensor.
 *   grad_ptrs  HOST array of W*n_tensors DEVICE pointers; entry k*n_tensors + l
 *              is worker k's gradient of tensor l (off[l+1]-off[l] floats, any
 *              4-byte alignment).  The library keeps the last four distinct tables
 *              on the device: a table seen before costs nothing, a new one is
 *              copied to the device with a blocking copy (and, once four are held,
 *              after a stream synchronisation, since the one it replaces may be
 *              in use).  While the stream is being captured into a HIP graph only
 *              a table that is already on the device is accepted (DEF_EINVAL
 *              otherwise: run one eager step with it first), and a table used under
 *              capture stays on the device, unchanged, until def_destroy, because
 *              every replay reads it.
 *   y_out      as in def_step (one flat vector of d floats) or NULL.
 * Works with either parameter mode.
 */
int def_step_tensors(def_ctx *ctx, const float *const *grad_ptrs, float *y_out);
int def_a_step_tensors(def_ctx *ctx, const float *const *grad_ptrs);

/*
 * One iteration in two halves, for deployments in which the workers are spread over
 * several GPUs (Sec. 5 "Settings": one worker per GPU, ring all-reduce): each GPU
 * holds W >= 1 of the workers and a replica of x, and the compressed blocks are
 * added across GPUs between the halves by a collective that the CALLER runs
 * (C is linear, Assumption 3.3, so the sum of blocks is the block of the sum).
 *
 *   def_pack   Algorithm 1 up to the all-reduce line for this GPU's W workers:
 *              momentum, error feedback, residual write-back (and the off-block
 *              detached points if set), then the sum over the local workers of
 *              their kept blocks,  block_sum[j] = sum_k C(p_k)[(s_t + j) mod d],
 *              k ascending from +0, NOT divided.  *block_sum (if block_sum is
 *              not NULL) receives the DEVICE address of that B-float vector,
 *              owned by the library (the same buffer def_state_ptrs calls
 *              avg_block); the caller may reduce it in place.  x is not touched.
 *              Every GPU must use the same seed, step counter, d and R, so that
 *              all draw the same block.  t <- t+1.
 *   def_apply  the update line: x[(s_t + j) mod d] -= block[j] / divisor for
 *              j < B, where block (DEVICE, B floats, may be *block_sum itself)
 *              is the caller's reduced vector and divisor the total number of
 *              workers over all GPUs; the in-block detached points (if set) and
 *              the averaged block seen through def_state_ptrs are written too.
 *              y_out as in def_step (with W local workers it subtracts the mean
 *              of the LOCAL error memories; with the same W on every GPU, DEF's
 *              y over all workers is the average of the GPUs' y_out, since all
 *              hold the same x: one more reduction of d floats by the caller,
 *              once, after training).
 *
 * def_pack followed by def_apply(*block_sum, W, y) on one GPU is bit-identical
 * to def_step.  A def_pack must be followed by def_apply before the next
 * def_pack or def_step (DEF_EINVAL otherwise, nothing changed); def_apply
 * without a preceding def_pack, or with divisor <= 0, is DEF_EINVAL.
 */
int def_pack(def_ctx *ctx, const float *grads, uint64_t ld, const float **block_sum);
int def_pack_tensors(def_ctx *ctx, const float *const *grad_ptrs, const float **block_sum);
int def_apply(def_ctx *ctx, const float *block, float divisor, float *y_out);

/*
 * DEF's output without stepping: y_out[i] = x[i] - (1/W) sum_k e_k[i] for the
 * current state (Algorithm 1 "Output").  y_out: DEVICE, d floats.
 */
int def_output(def_ctx *ctx, float *y_out);

/*
 * Detached evaluation points (Algorithm 1, "detach" line; Sec. 3.2): worker k
 * computes its next gradient at  w_k = x - lambda * e_k,  lambda in [0, 1]
 * (0.3 in the paper's experiments; lambda = 0 is plain error feedback).
 *
 * def_set_detach  from now on every step also writes, in the same pass,
 *                 w_out[k*ldw + i] = x_{t+1}[i] - lambda * e_{k,t+1}[i]
 *                 for all workers k and indices i.  w_out: DEVICE, [W][ldw] floats,
 *                 ldw >= d, caller-owned, must stay valid while set.
 *                 w_out == NULL switches it off.  The call itself writes the
 *                 points of the current state (as def_detach does), so w_out is
 *                 valid at once: before the first step it holds x_0 in every row
 *                 (e_{k,0} = 0).  Not allowed between def_pack and def_apply
 *                 (DEF_EINVAL).
 * def_detach      writes the same quantity for the CURRENT state (after a restore,
 *                 or with another lambda) without stepping.
 * DEF_EINVAL for lambda outside [0, 1], ldw < d, or a misaligned pointer.
 */
int def_set_detach(def_ctx *ctx, float *w_out, uint64_t ldw, float lambda);
int def_detach(def_ctx *ctx, float *w_out, uint64_t ldw, float lambda);

/*
 * Error-memory statistics of the current state (Sec. 3.2, items (1)-(3) and
 * Eq. (9); Appendix A, first display), accumulated in float64.  With
 * e_t = (1/W) sum_k e_k:
 *   out[0] = ||e_t||^2                       the distance ||x_t - y_t||^2 of plain EF
 *   out[1] = (1/W) sum_k ||e_k||^2
 *   out[2] = lambda*(t) = out[0] / out[1]    (0 if out[1] is 0)
 *   out[3] = (1/W) sum_k ||e_t - lambda*e_k||^2   DEF's average distance at lambda
 * out: DEVICE, 4 doubles, 8-byte aligned.  Asynchronous like a step; reproducible
 * from run to run (no atomics).  DEF_EINVAL for lambda outside [0, 1].
 */
int def_diagnostics(def_ctx *ctx, float lambda, double *out);

/*
 * def_diagnostics for callers that cannot allocate device memory and have no context:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It computes the same four numbers from error memories the CALLER holds
 * (a checkpoint it restored itself, or the views of def_state_ptrs) and allocates
 * nothing, not even at its first call: the per-workgroup partial sums live in a
 * fixed 4 MiB array inside the library's device image, one copy per GPU, kept until
 * the process ends.
 *   e       DEVICE, read-only: worker k's error memory at e + k*ld, d floats used;
 *           16-byte aligned, ld >= d and a multiple of 4.  Columns d..ld-1 are not read.
 *   d, W    as in def_config; d <= DEF_STATIC_MAX_D, else DEF_ELIMIT (nothing is run).
 *   lambda  in [0, 1].
 *   out     DEVICE, 4 doubles as def_diagnostics writes them, 8-byte aligned.
 *   stream  hipStream_t of the GPU that is current in the calling thread (NULL = the
 *           null stream); only two kernel launches are enqueued, no memset, no copy.
 * Every call on a GPU uses that GPU's one array (fully overwritten as far as it is
 * read, so nothing needs clearing): calls that overlap in time on one GPU, on different
 * streams, race with each other; calls on one stream, or on different GPUs, do not.
 * Results are bit-identical to def_diagnostics on the same error memories.
 */
#define DEF_STATIC_MAX_D ((uint64_t)268435456)   /* 2^19 doubles / 2 per 1024 columns */
int def_diagnostics_static(const float *e, uint64_t ld, uint64_t d, uint32_t W, float lambda, double *out,
                           void *stream);

/*
 * The same per worker (Sec. 3.2, item (1); Appendix A, first display): for
 * k = 0..W-1, with e_t = (1/W) sum_k e_k,
 *   out[k]       = ||e_k||^2
 *   out[W + k]   = <e_t, e_k>
 *   out[2W + k]  = lambda*(k,t) = <e_t, e_k> / ||e_k||^2   (0 if e_k = 0): the lambda at
 *                  which worker k's point x - lambda*e_k is closest to y_t.
 * out: DEVICE, 3*W doubles, 8-byte aligned.  Asynchronous; float64 sums in a fixed
 * order (no atomics).  (1/W) sum_k out[W + k] equals def_diagnostics' out[0].
 */
int def_diagnostics_workers(def_ctx *ctx, double *out);

/* Replace the seed (Sec. 1: the seed all workers share).  t keeps counting. */
int def_set_seed(def_ctx *ctx, uint64_t seed);

/*
 * Block draw on the device, for callers that capture steps into a HIP graph.
 *
 * By default the start index of a step is drawn on the host when the step is
 * enqueued and travels as a kernel argument, so a captured step would replay the
 * same block for ever.  With the device draw switched on, every step begins with
 * a one-thread kernel that draws s_t from a device-resident copy of (seed, t) -
 * the same Philox4x64-10 draw - advances t there and hands s_t to the other
 * kernels through device memory.  A captured step (or run of steps) can then be
 * replayed: each replay performs the next iteration(s).  A step enqueues only
 * kernel launches (no memset, no copy, no allocation, no synchronisation), so it
 * can be captured with hipStreamBeginCapture on the context's stream; gradients
 * are read from the addresses given at capture time, and eta, lambda and the
 * output pointers are captured by value (capture again after def_set_lr).  Do not
 * profile (def_profile_begin) while capturing.
 *
 * def_set_device_draw  on != 0: copy the host's (t, seed, pending forced start)
 *                      to the device and use the device draw from the next step;
 *                      on == 0: back to the host draw (call def_sync_step first if
 *                      graphs were replayed).  def_set_seed, def_set_step and
 *                      def_force_next_start keep working: in this mode they also
 *                      enqueue a one-thread kernel that updates the device copy.
 * def_sync_step        replays advance t on the device only.  This call copies the
 *                      device's t (and the start of the last step) back so that
 *                      def_get_step and def_last_block are current again.
 *                      Synchronises the stream; not allowed during capture.
 */
int def_set_device_draw(def_ctx *ctx, int on);
int def_sync_step(def_ctx *ctx);

/* Learning-rate schedules (eta = c/(t+1) in Theorem 4.6; step decay in Sec. 5 "Settings"). */
int def_set_lr(def_ctx *ctx, float lr);

/* Step counter, for resuming: the state of a run is (x, e, m, seed, t, eta). */
int def_set_step(def_ctx *ctx, uint64_t t);
int def_get_step(const def_ctx *ctx, uint64_t *t);

/*
 * Use start index s (0 <= s < d) for the NEXT step only instead of the seeded
 * draw; s < 0 clears a pending request.  For tests and for workloads that force
 * a block across the end of the vector.
 */
int def_force_next_start(def_ctx *ctx, int64_t s);

/* Start index and length B of the block kept by the most recent step. */
int def_last_block(const def_ctx *ctx, uint64_t *start, uint64_t *len);

/* Block length B = ceil(d/R) of this context (delta = B/d, Assumption 4.2). */
int def_block_length(const def_ctx *ctx, uint64_t *len);

/*
 * The shared block draw as a pure function (HOST, no GPU needed):
 *   *start = Philox4x64-10(counter = (t,0,0,0), key = (seed,0))[0] mod d.
 * (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3", SC 2011.)
 */
int def_block_start(uint64_t seed, uint64_t t, uint64_t d, uint64_t *start);

/*
 * DEVICE views of the library-owned state, for checkpoints and parity checks.
 *   *e, *m       [W][*ld_state] floats, worker k's row at + k * *ld_state, column i
 *                = flat parameter index i; *ld_state >= d (a multiple of 256);
 *                columns d..ld_state-1 are padding and stay zero.
 *                *m is NULL when momentum == 0.
 *   *avg_block   B floats: the averaged block C(p_t) of the last step in compact
 *                form, entry j belongs to flat index (start + j) mod d.
 * Any out-pointer may be NULL.  The views stay valid until def_destroy; writing
 * through e/m (restoring a checkpoint) is allowed between steps.
 */
int def_state_ptrs(def_ctx *ctx, float **e, float **m, float **avg_block, uint64_t *ld_state);

/* How the last step addressed its inputs: 1 = flat gradient buffer (and flat x if the pass
 * reads x), 0 = per-tensor pointers resolved through the offset table. */
int def_last_path(const def_ctx *ctx, int *flat);

/*
 * Name and launch shape of the streaming kernel the last step ran, e.g.
 * "def_stream_vec4_kernel<mu=1,wd=1,detach=0,threads=64,...>".
 * For profiles and benchmarks that must say exactly which kernel they measured.
 * The string is owned by the context and valid until the next step or def_destroy;
 * NULL if no step has run.
 */
const char *def_last_kernel(const def_ctx *ctx);

/*
 * Per-launch timing of the streaming kernel (the fused momentum + error
 * feedback + residual pass, which moves nearly all of a step's bytes), with HIP
 * events recorded on the context's stream immediately before and after that
 * launch.
 *   def_profile_begin  allocates max_steps event pairs; the next max_steps steps
 *                      each record one pair (later steps are not recorded).
 *   def_profile_end    waits for the last recorded event, writes up to cap
 *                      durations in milliseconds to ms (HOST), stores the
 *                      number recorded in *n, and frees the events.
 */
int def_profile_begin(def_ctx *ctx, uint32_t max_steps);
int def_profile_end(def_ctx *ctx, float *ms, uint32_t cap, uint32_t *n);

/* Text for a def_status; HIP error code of the last DEF_EHIP (0 if none). */
const char *def_strerror(int status);
int def_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DEF_H_ */
