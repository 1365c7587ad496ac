/*
 * pier.h - C ABI of the MI355X (gfx950) implementation of the optimizer hot path
 * of Pier's two-level optimizer: the inner AdamW step of every group replica, the
 * outer Nesterov step with momentum warmup / momentum decay, and the host-offload
 * stream for the outer state.
 *
 * Notation (the paper's): theta_g = model of group g, G groups; theta_{t-r} = the
 * model at the previous synchronisation, here "anchor"; M = outer momentum;
 * r = synchronisation interval; T = training iterations; mu = momentum coefficient.
 *
 * Conventions
 *  - Every function returns a pier_status and never throws or aborts across the
 *    ABI; pier_last_error() gives the reason of the calling thread's last failure.
 *  - All argument checks happen before anything is enqueued: a call that returns an
 *    error has launched nothing and changed no buffer (pier_train_step included: on a
 *    synchronisation iteration the outer step's arguments are checked before the first
 *    inner launch).  The only errors that can follow a launch are failures the HIP
 *    runtime reports while enqueueing (PIER_ERR_HIP).
 *  - Threads: a context is not synchronised internally.  Calls on DIFFERENT contexts may
 *    run concurrently from different threads; calls on ONE context - bind calls and
 *    launches alike - must be serialised by the caller.  pier_last_error() is per thread.
 *    The host-only helpers (schedules, pier_placement_plan, pier_status_string) are
 *    re-entrant.
 *  - "device pointer" = memory of the GPU that was current when the context first
 *    touched the GPU (first bind call); the caller keeps that device current for
 *    every later call.  Bind calls verify that numel elements starting at each pointer
 *    lie inside the HIP allocation the pointer belongs to (PIER_ERR_INVALID_ARG
 *    otherwise).  The check is per underlying allocation: for a pointer handed out by a
 *    sub-allocator (PyTorch's caching allocator) it bounds that allocator's segment, not
 *    the tensor.  "host pointer" = ordinary host memory unless "pinned" is said.
 *  - Ownership: the caller owns all parameter, state, gradient, staging and pinned
 *    memory and all streams.  The library owns only small tables (pointer lists,
 *    chunk lists, events) that live as long as the context.
 *  - Kernels and copies are enqueued on the caller's streams; calls do not
 *    synchronise unless stated.  hip_stream arguments are hipStream_t values passed
 *    as void* (NULL = the null stream).  Once a context's tensors are bound, the launch
 *    calls (pier_inner_adamw, pier_inner_adamw_clipped[_static], pier_outer_step and a
 *    resident pier_train_step) enqueue kernels and nothing else - no allocation, no
 *    memset, no copy, no synchronisation - so a caller may record them into a HIP graph.
 *    Scalars (step, learning rates, mu) travel as kernel arguments and are fixed in a
 *    recorded graph.
 *  - All model-sized buffers are fp32, updated in place.  A model is a list of
 *    n_tensors separately allocated tensors; tensor i has numel[i] elements.  A
 *    pointer must be aligned to its element size; 16-byte aligned tensors take the
 *    128-bit path, others a slower scalar path with identical results.
 *  - Results are deterministic: they do not depend on chunking, grid size, or the
 *    offload chunk size; the sum over groups always runs g = 0, 1, ..., G-1.
 */
#ifndef PIER_H
#define PIER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PIER_OK = 0,
    PIER_ERR_INVALID_ARG = 1, /* null / negative / out-of-range argument            */
    PIER_ERR_ALIGNMENT = 2,   /* pointer not aligned to its element size            */
    PIER_ERR_STATE = 3,       /* call made before the bindings it needs             */
    PIER_ERR_OOM = 4,         /* a table or event could not be allocated            */
    PIER_ERR_HIP = 5          /* the HIP runtime reported an error (text in last_error) */
} pier_status;

/* Version of this interface: PIER_ABI_VERSION of the header the library was built from.
 * It changes whenever a declared function, struct or enum changes incompatibly. */
#define PIER_ABI_VERSION 3
int pier_abi_version(void);

/* Text of the calling thread's most recent error; never NULL; valid until the
 * thread's next failing call. */
const char* pier_last_error(void);
/* Name of a status code ("PIER_OK", ...); never NULL. */
const char* pier_status_string(pier_status s);

/* ----------------------------------------------------------------- context */

typedef struct pier_ctx pier_ctx; /* opaque */

/* Describes the model: n_tensors >= 1 tensors with numel[i] >= 0 elements (host
 * array, copied), held by n_replicas >= 1 group replicas (at most
 * PIER_MAX_REPLICAS).  Host-only: touches no GPU. */
#define PIER_MAX_REPLICAS 64
pier_status pier_ctx_create(pier_ctx** out, int n_tensors, const int64_t* numel, int n_replicas);
/* Frees the library's tables and events.  Caller buffers are not touched.  The
 * caller must have drained the streams it used with this context. */
pier_status pier_ctx_destroy(pier_ctx* ctx);
/* Sum of numel (the parameter count N); -1 if ctx is NULL. */
int64_t pier_ctx_numel(const pier_ctx* ctx);

/* Launch shape of the kernels; defaults suit MI355X and results never depend on it.
 * chunk_elems: elements one workgroup handles per chunk (multiple of 1024, >= 1024);
 * unroll: 128-bit loads each lane keeps in flight per stream (1, 2 or 4);
 * max_grid: cap on workgroups per launch (0 = no cap: one chunk per workgroup; always
 * taken as given); nontemporal: 1 = mark loads/stores as streaming.  chunk_elems = 0,
 * unroll = 0, nontemporal = -1 keep that field unchanged.  Must be called before the
 * first bind. */
pier_status pier_ctx_set_launch(pier_ctx* ctx, int64_t chunk_elems, int unroll, int max_grid,
                                int nontemporal);

/* Optional: how many wavefronts the kernels keep resident (tuning only, results do not
 * change).  wg_threads: 256 = one four-wave workgroup per chunk, 64 = four one-wave
 * workgroups per chunk (then one vector per lane per stream, whatever `unroll` says),
 * 0 = each kernel's measured best (64 unless unroll or max_grid were set);
 * lds_bytes: LDS reserved per workgroup and left unused, which caps the workgroups a
 * compute unit holds at floor(160 KiB / lds_bytes) (0 = no cap; at most 65536),
 * -1 = each kernel's measured best (12 waves per compute unit for the AdamW step, 8
 * for the outer step, 20 for the lazy-start synchronisation).  Default: 0, -1.  May be called at any time between launches. */
pier_status pier_ctx_set_occupancy(pier_ctx* ctx, int wg_threads, int lds_bytes);

/* Optional: how many workgroups, hence partial sums, the gradient-norm pass of the clipped
 * step folds (1 .. 2^20; 0 = the default, 16384; a model with fewer chunks uses one per
 * chunk).  The fold order, and with it the last bits of the norm, follow this number.
 * Must be called before the first bind. */
pier_status pier_ctx_set_norm_fold(pier_ctx* ctx, int n_partials);

/* Binds replica `replica` (0-based).  p, m, v, grad are HOST arrays of n_tensors
 * DEVICE pointers: parameters theta_g, AdamW first and second moments (fp32), and
 * the gradient of each tensor, fp32 or (grad_is_bf16 != 0) bfloat16.  A tensor with
 * numel 0 may have NULL pointers.  May be called again to re-point a replica: the
 * tables are rewritten with a synchronous small copy, so no launch of this context
 * may be in flight during a re-bind (the same holds for pier_bind_outer). */
pier_status pier_bind_replica(pier_ctx* ctx, int replica, float* const* p, float* const* m,
                              float* const* v, const void* const* grad, int grad_is_bf16);

/* Optional bfloat16 working copy of replica `replica`'s parameters (section
 * "Experiments": BF16 in models, FP32 in optimizers).  w_bf16 is a HOST array of
 * n_tensors DEVICE pointers to 2-byte elements, or NULL to unbind.  Once bound, every
 * step that writes theta_g (pier_inner_adamw[_clipped]; the Pier phase of the outer
 * step, resident or offloaded) also writes bfloat16(theta_g) there, rounded to nearest
 * even (NaN -> 0x7FC0), in the same pass (+2 B/param written).  The outer step needs
 * the working copies of all replicas bound, or of none.  Needs the replica bound. */
pier_status pier_bind_shadow(pier_ctx* ctx, int replica, uint16_t* const* w_bf16);

typedef enum {
    PIER_LOC_DEVICE = 0,     /* anchor[i], momentum[i]: device pointer of tensor i      */
    PIER_LOC_HOST_PINNED = 1 /* anchor[0], momentum[0]: one flat PINNED host array each,
                                N floats, tensors back to back in list order          */
} pier_loc;
/* Binds the outer optimizer's state: the anchor theta_{t-r} and the momentum M.
 * The arrays `anchor` / `momentum` themselves are host arrays (n_tensors entries
 * for DEVICE, 1 entry for HOST_PINNED). */
pier_status pier_bind_outer(pier_ctx* ctx, pier_loc loc, float* const* anchor,
                            float* const* momentum);

/* ------------------------------------------------------- inner AdamW step
 * One AdamW update of replica `replica` (Algorithm 1 / Algorithm 2,
 * "OptimizerUpdate"; section "Implementation": AdamW inside each group; Table I).
 * Per element, in fp32:
 *     g  = grad * grad_scale
 *     m  = beta1 m + (1 - beta1) g          v = beta2 v + (1 - beta2) g^2
 *     mh = m / (1 - beta1^step)             vh = v / (1 - beta2^step)
 *     theta = theta - lr * ( mh / (sqrt(vh) + eps) + weight_decay * theta )
 * step >= 1 is the global iteration count (moments are never reset by an outer step).
 * One kernel launch over the whole tensor list on `hip_stream`. */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float grad_scale; /* 1 on the plain path; multiplies every gradient element */
    int64_t step;
} pier_adamw_hp;
pier_status pier_inner_adamw(pier_ctx* ctx, int replica, const pier_adamw_hp* hp, void* hip_stream);

/* The same step preceded by global-norm gradient clipping (Table I: "clip grad 1"; the
 * paper names the threshold, the rule is the usual one): over all gradient elements of
 * the replica, norm = sqrt(sum g^2) accumulated in double, coefficient
 * c = min(1, max_norm / (norm + 1e-6)) rounded to fp32, and the step runs with every
 * gradient element multiplied by grad_scale * c.  Three launches on hip_stream (partial
 * sums, fold, AdamW), no host synchronisation; the gradient is read twice (32 B/param).
 * The fold uses a fixed order, so the norm is the same in every run. */
pier_status pier_inner_adamw_clipped(pier_ctx* ctx, int replica, const pier_adamw_hp* hp,
                                     float max_norm, void* hip_stream);
/* For callers that cannot allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): pier_inner_adamw_clipped with the norm pass's scratch -
 * its per-workgroup partial sums and its 24-byte norm/coefficient record - in a static
 * device array of 131 328 bytes (256 + 8 x 16384) that each GPU holds until the process
 * ends, instead of in buffers of the context.  The call allocates and frees nothing (the
 * array's address was resolved when the context first bound a tensor) and clears
 * nothing: every word of scratch it reads it has written itself.  Same launches, same
 * arguments, same results bit for bit as pier_inner_adamw_clipped.
 * PIER_ERR_INVALID_ARG when the context's norm pass folds more than 16384 partial sums
 * (pier_ctx_set_norm_fold), which the array does not hold; nothing is launched then.
 * ALL calls on one GPU - any context, any replica, any stream - share that GPU's array:
 * two such calls that overlap in time race on it, so the caller keeps them on one stream
 * or orders them with events.  pier_grad_norm_last after this call reads the array, and
 * is valid only until the next call of this function on the same GPU. */
pier_status pier_inner_adamw_clipped_static(pier_ctx* ctx, int replica, const pier_adamw_hp* hp,
                                            float max_norm, void* hip_stream);

/* Norm and coefficient computed by the replica's most recent clipped step: waits for
 * hip_stream, then copies them to the host (either output may be NULL). */
pier_status pier_grad_norm_last(pier_ctx* ctx, int replica, double* norm_out, float* coef_out,
                                void* hip_stream);

/* ----------------------------------------------------------- outer step
 * One kernel launch, with anchor and M on the device.
 *   PIER (Algorithm 2's synchronisation branch), over all replicas:
 *     delta = (1/G) sum_g (theta_g - anchor)          [the all-reduce's arithmetic]
 *     M     = mu M + delta
 *     theta = anchor + outer_lr (mu M + delta); anchor = theta_g = theta for all g
 *     (8G + 16 bytes per parameter)
 *   WARMUP (Algorithm 1's, the lazy-start phase).  That algorithm has ONE model - the
 *     groups are formed after it - so the model is read from replica 0; the caller
 *     keeps the replicas identical in this phase (synchronised data parallelism):
 *     delta = theta_0 - anchor;  M = mu M + delta;  anchor = theta_0  (bit for bit)
 *     replicas and their AdamW state untouched; outer_lr ignored
 *     (20 bytes per parameter whatever G)
 * M holds the paper's sign (it accumulates new - old).  Needs every replica bound
 * and pier_bind_outer(PIER_LOC_DEVICE). */
typedef enum { PIER_PHASE_WARMUP = 0, PIER_PHASE_PIER = 1 } pier_phase;
typedef struct {
    float outer_lr, mu;
    pier_phase phase;
} pier_outer_hp;
pier_status pier_outer_step(pier_ctx* ctx, const pier_outer_hp* hp, void* hip_stream);

/* ------------------------------------------------- host-offload outer step
 * The same outer step with anchor and M resident in pinned host memory (section
 * "Implementation": the previous model and the outer momentum are offloaded to the
 * host, reloaded at the start of the outer step and written back at its end).  The
 * flat index space is cut into pieces of chunk_bytes (multiple of 16; 256 MiB is the
 * intended size); piece k is copied host->device on h2d_stream, processed by the
 * outer kernel on compute_stream and copied back on d2h_stream, the three stages of
 * different pieces overlapping.  `workspace` is caller-owned device memory holding
 * the staging slots (2 arrays x chunk_bytes per slot; 1 to 64 slots are used, 3
 * recommended = pier_offload_workspace_bytes).  Results are bit-identical to
 * pier_outer_step.  compute_stream is made to wait for the last copy-back, so work
 * enqueued on it afterwards sees both the replicas and the host arrays complete; the
 * call itself returns after enqueueing unless `stats` is non-NULL, in which case it
 * waits for completion and fills the timings (milliseconds, bytes; *_ms are the
 * summed durations of that stage's operations, wall_ms first copy-in to last
 * copy-back).  The three streams must be distinct for overlap but need not be.
 * Needs pier_bind_outer(PIER_LOC_HOST_PINNED).  The first call with a new
 * chunk_bytes builds and uploads that chunking's tables (a small synchronous copy). */
typedef struct {
    double h2d_bytes, d2h_bytes, h2d_ms, d2h_ms, kernel_ms, wall_ms;
    int n_pieces, n_slots;
    double compute_ms; /* first reload to last kernel: what compute_stream waits for in trailing mode */
} pier_offload_stats;
pier_status pier_offload_workspace_bytes(const pier_ctx* ctx, size_t chunk_bytes, size_t* out);
/* When the write-back may finish.  trailing = 0 (default): as described above,
 * compute_stream waits for the last copy-back.  trailing = 1: it does not - the replicas
 * are final when compute_stream has passed the call's kernels, so the next inner steps
 * start while the copy-back still runs; the host arrays and the workspace are final when
 * d2h_stream has drained, and the caller leaves both alone until then (the next
 * pier_offload_stream call waits for it by itself).  Pays off when the workspace holds
 * enough slots for the reload to run ahead of the slower copy-back (up to 64 are used;
 * about 7 GB of backlog builds up over the 7B model's 53 GB).  Results do not change. */
pier_status pier_ctx_set_offload_writeback(pier_ctx* ctx, int trailing);
pier_status pier_offload_stream(pier_ctx* ctx, const pier_outer_hp* hp, size_t chunk_bytes,
                                void* workspace, size_t workspace_bytes, void* compute_stream,
                                void* h2d_stream, void* d2h_stream, pier_offload_stats* stats);

/* --------------------------------------------------------- placement probe
 * Not an operation of the paper: a measurement aid for laying the caller's buffers out
 * in MI355X's HBM.  The two kernels stream several buffers in place at once, and the
 * rate they sustain depends on where those buffers sit relative to each other: the
 * 288 GiB behave as three classes of 96 GiB (buffers streamed together from different
 * classes reach ~6.5 TB/s, from one class ~6.0 TB/s).  This call classifies the
 * n_granules consecutive granules of granule_bytes (multiple of 2 MiB, >= 512 MiB)
 * that start at the device pointer `arena`, by timing a two-buffer in-place streaming
 * pass between granules: class_out[g] (host array) receives a small class id, equal for
 * granules that behave as one class.  A caller then places the buffers that one launch
 * touches together as pier_placement_plan says.  Synchronous (a few seconds); OVERWRITES
 * the arena's contents;
 * enqueues on hip_stream and waits for it. */
pier_status pier_hbm_probe(void* arena, size_t bytes, size_t granule_bytes, int32_t* class_out,
                           int n_granules, void* hip_stream);

/* The classification step of the probe on its own (pure host arithmetic, touches no GPU):
 * rates is a host array of n_granules x n_granules positive numbers, rates[a * n_granules + b]
 * = the streaming rate of granules a and b together, in any unit; class_out as above.  Every
 * threshold is a fraction of the best rate in the table: a pairing counts as "different
 * classes" when it is within 3.3 % of the best rate; the arena counts as several classes
 * only if at least 15 % of a sweep of granules are that fast against BOTH of granules 0 and
 * 1 and the next slower sample lies at least 2 % of the best rate below them.  pier_hbm_probe
 * is this routine fed with rates it measures on demand (a few hundred of the n^2 pairs). */
pier_status pier_hbm_classify(const double* rates, int n_granules, int32_t* class_out);

/* What the calling thread's most recent pier_hbm_probe (or pier_hbm_classify) saw: the
 * fastest pairing (for the probe: TB/s of a two-buffer in-place streaming pass with
 * trivial arithmetic, i.e. what this GPU gives the access pattern of the two optimizer
 * kernels at best), the level a pairing had to reach to count as "different classes"
 * (0 when the arena is one class), the number of classes and of pairings asked for.  Any
 * output may be NULL.  PIER_ERR_STATE before the thread's first probe. */
pier_status pier_hbm_probe_summary(double* best_rate, double* threshold, int32_t* n_classes,
                                   int32_t* n_pairs);

/* The placement that goes with the probe (again no operation of the paper; host
 * arithmetic only, touches no GPU).  Measured on MI355X: a launch streams fastest when
 * its buffers lie in exactly two classes, half in each.  For a model with n_replicas
 * replicas this returns the class of every model-sized buffer:
 *   theta_g and m_g           class g mod 2;
 *   anchor, momentum          (outer_on_device != 0) whichever of classes 0 and 1 then holds
 *                             fewer of the outer step's n_replicas + 2 buffers;
 *   v_g and grad_g            class 2 while the pair fits there, else the class of {0, 1}
 *                             that theta_g is not in (shared_grad != 0: one gradient
 *                             buffer for all replicas, placed with replica 0's v).
 * room[c] (host array of n_classes entries) is the number of buffers of this model that
 * class c still holds; a full class passes its buffer on to the next class on its list,
 * then to the class with most room.  With one or two classes the same rules apply modulo
 * the class count.  The caller should allocate in the order the plan was made - theta_0,
 * m_0, theta_1, m_1, ..., anchor, momentum, v_0, grad_0, v_1, ... - so that buffers that
 * are streamed together also end up next to each other inside a class.
 * replicas: host array of n_replicas entries (out); anchor_class, momentum_class: out,
 * -1 when outer_on_device == 0.  PIER_ERR_OOM when the buffers do not fit room[]. */
typedef struct {
    int32_t theta, m, v, grad;
} pier_replica_placement;
pier_status pier_placement_plan(int n_classes, const int64_t* room, int n_replicas, int shared_grad,
                                int outer_on_device, pier_replica_placement* replicas,
                                int32_t* anchor_class, int32_t* momentum_class);

/* ------------------------------------------------------------- schedules
 * Pure host helpers; t = iteration (1-based), T = total iterations (> 0). */

/* Algorithm 2's momentum-decay choice: 0.99 for 0.1T <= t < 0.15T, 0.95 for
 * 0.15T <= t < 0.2T, 0.9 otherwise (breakpoints compared in integers). */
float pier_mu_schedule(int64_t t, int64_t T);
/* Section "Implementation": 0 below 0.1T, linear 0 -> 1 on [0.1T, 0.2T), 1.1 on
 * [0.2T, 0.8T), 0.9 on [0.8T, T]. */
float pier_outer_lr_schedule(int64_t t, int64_t T);
/* Fills the scalars of the synchronisation at iteration t: lazy-start phase
 * (t <= 0.1T, Algorithm 1's inclusive loop bound) -> WARMUP with Algorithm 1's
 * default mu = 0.9; afterwards PIER with the two schedules above. */
pier_status pier_outer_schedule(int64_t t, int64_t T, pier_outer_hp* out);

/* Inner learning rate (Table I: cosine decay, 2 % warmup, minimum learning rate, decay
 * iterations = T): lr_max * t / W for t <= W = warmup_frac * T, then half a cosine from
 * lr_max at W to lr_min at T (lr_min beyond).  Evaluated in double, rounded to fp32. */
float pier_inner_lr_schedule(int64_t t, int64_t T, float lr_max, float lr_min, double warmup_frac);

/* -------------------------------------------------------- one training iteration
 * Algorithm 2's loop body for iteration t (1-based) as one call, for a caller that has
 * just put the gradients of every replica in the bound gradient tensors: the inner
 * AdamW step of every replica with the scheduled learning rate (preceded by global-norm
 * clipping when clip_norm > 0), and, when t is a multiple of r, the outer step with the
 * scalars of pier_outer_schedule (mode PIER) or with DiLoCo's fixed outer learning rate
 * 0.7 and momentum 0.9 and no lazy-start phase (mode DILOCO: the baseline the paper
 * compares with).  The outer step runs resident or, when anchor and M are bound as
 * pinned host arrays, through pier_offload_stream with the workspace and side streams
 * given here.  (The paper's listing prints the inner step only for t mod r != 0; as in
 * Algorithm 1 the step is taken every iteration.)  Everything is enqueued on
 * `hip_stream` (plus the side streams); nothing synchronises. */
typedef enum { PIER_MODE_PIER = 0, PIER_MODE_DILOCO = 1 } pier_mode;
typedef struct {
    int64_t T;                 /* training iterations                                  */
    int64_t r;                 /* synchronisation interval                             */
    pier_mode mode;
    float lr_max, lr_min;      /* inner learning-rate schedule                         */
    double warmup_frac;        /* 0.02 in Table I                                      */
    float beta1, beta2, eps, weight_decay;
    float clip_norm;           /* > 0: clipping threshold (Table I: 1); 0: no clipping */
    size_t chunk_bytes;        /* offload only                                         */
    void* workspace;           /* offload only: device staging memory                  */
    size_t workspace_bytes;
    void* h2d_stream;          /* offload only                                         */
    void* d2h_stream;
} pier_train_cfg;
pier_status pier_train_step(pier_ctx* ctx, const pier_train_cfg* cfg, int64_t t, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PIER_H */
