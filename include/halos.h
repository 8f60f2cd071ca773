/*
 * halos.h -- C ABI of the HALoS server-side update path on one AMD GPU.
 *
 * HALoS (arXiv 2506.04531) trains with a two-level parameter-server hierarchy:
 * local parameter servers (LPS) apply worker deltas with a momentum step and
 * accumulate them, a global parameter server (GPS) applies the accumulated
 * updates with its own momentum step, and each LPS merges the returned global
 * model into its local model (Algorithm 1; update rule in Appendix E).  This
 * library is that server side, over a list of parameter tensors that all live
 * in one GPU's memory.  Each call below is one message or one step of
 * Algorithm 1.
 *
 * Conventions
 *   Pointers     "device" pointers are GPU addresses, "host" pointers are CPU
 *                addresses.  Pointer ARRAYS (void *const *) are host arrays of
 *                n_tensors device pointers, one per tensor of the layout.
 *   Layout       tensor i is a contiguous array of numel[i] elements; every
 *                non-empty tensor's base address must be 16-byte aligned.
 *                Server state is fp32 (the momentum arrays optionally bfloat16, HALOS_FLAG_BF16_MOMENTUM).
 *                Worker deltas are fp32, bfloat16 or IEEE half (or arrive as the worker's fp32 end model,
 *                halos_lps_push_end_model).
 *   Ownership    all parameter-sized buffers are allocated by the caller and
 *                only BORROWED: state buffers for the life of the handle, a
 *                pushed delta until the step that consumes it has finished on
 *                its stream, a pull destination until that copy has finished.
 *                The library allocates only small tables and frees them in the
 *                destroy calls.  It never frees caller memory.
 *                A set of delta / destination pointers is checked against its allocations
 *                (device memory, alignment, room for every tensor) the first time a server
 *                sees it and trusted while the same addresses keep coming; a caller that
 *                frees such a buffer and later passes another allocation at the same
 *                address calls halos_forget_buffers first.
 *   Streams      `stream` is a hipStream_t (NULL = the default stream).  Device
 *                work is enqueued there and the call returns; the caller
 *                synchronises.  All calls that touch the same server's state
 *                must be issued on streams that are ordered with each other.
 *   Graphs       the event-loop calls (push_update / push_end_model with a pointer
 *                set the worker has used before, push_global, step, step_pull, step_batch,
 *                step_average, gps_merge, pull_model with a destination used before) only launch
 *                kernels on `stream`: no allocation, no synchronisation, no memset.
 *                They may therefore be issued on a capturing stream.  Host-side
 *                protocol state advances when a call is made, not when a graph is
 *                replayed, so only a sequence that brings the protocol back to its
 *                starting state (a whole accumulation cycle) can be replayed as is.  step_batch
 *                and step_average keep, per worker, a device table of its delta pointers and
 *                rewrite it (a small kernel on `stream`) only when the worker shows another
 *                buffer: a graph holding them is replayed from the table state it was captured
 *                in (capture after one warm-up cycle; no batch calls with other buffers between
 *                replays).
 *   Threads      a handle may be used by one host thread at a time; creating or
 *                destroying an LPS, and halos_gps_merge, also count as a use of its GPS.
 *   Errors       every call returns a halos_status; on anything but HALOS_OK no
 *                host or device state has been modified and halos_last_error()
 *                describes the problem (thread-local string).  The one
 *                exception is HALOS_EHIP out of a step on a tensor list so long
 *                that it needs several launches: earlier launches of that step
 *                may already have run.
 *   Sign         a "delta" handed to this library is the PSEUDO-GRADIENT
 *                g = (model the sender started from) - (model it ended with),
 *                i.e. the negative of Algorithm 1's delta / Delta, so that
 *                beta = 0, eta = 1 adopts the sender's progress.
 */
#ifndef HALOS_H
#define HALOS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct halos_gps halos_gps;   /* opaque: global parameter server */
typedef struct halos_lps halos_lps;   /* opaque: local parameter server  */

typedef enum {
    HALOS_OK = 0,
    HALOS_EINVAL = 1,   /* bad argument: null/misaligned pointer, bad size, bad hyper-parameter */
    HALOS_ESTATE = 2,   /* call not allowed in the current protocol state */
    HALOS_ENOMEM = 3,   /* a small table could not be allocated */
    HALOS_EHIP = 4      /* the HIP runtime reported an error */
} halos_status;

/* Element type of a worker delta.  bfloat16 and IEEE half (the paper's workers train in fp16, Sec. 5.1) are upcast
 * exactly inside the update pass. */
#ifdef __cplusplus     /* a C++ caller or the library itself: every int32 value may arrive, an unknown one is answered with EINVAL */
typedef enum halos_dtype : int32_t { HALOS_F32 = 0, HALOS_BF16 = 1, HALOS_F16 = 2 } halos_dtype;
#else
typedef enum { HALOS_F32 = 0, HALOS_BF16 = 1, HALOS_F16 = 2 } halos_dtype;
#endif

/* Tensor list.  numel is a host array, copied by the create call. */
typedef struct {
    int32_t n_tensors;
    const int64_t *numel;
} halos_layout;

/* ModelUpdate(x, g, eta, beta) of Algorithm 1, as defined in Appendix E:
 *     m <- beta * m + g
 *     x <- x - eta * (cg * g + beta * m)
 * The paper's rule has cg = 1 - beta; cg = 1 is the textbook Nesterov step.
 * halos_*_set_momentum_delay switches a server to the delayed form of the same rule. */
typedef struct {
    float eta;
    float beta;
    float cg;
} halos_rule;

/* The paper's rule for a rate and a momentum coefficient: cg = 1 - beta, formed in fp32 (App. E). */
halos_rule halos_paper_rule(float eta, float beta);

/* Hyper-parameters of Algorithm 1 (its REQUIRE line). */
typedef struct {
    halos_rule local;    /* eta_l, beta_l: used by every LPS                       */
    halos_rule global;   /* eta_g, beta_g: used by the GPS                         */
    float alpha;         /* merge weight of the global model, 0 <= alpha <= 1      */
    int32_t K;           /* local updates accumulated before a Delta is sent, >= 1 */
    uint32_t flags;      /* HALOS_FLAG_* bits; all others must be 0                */
} halos_hparams;

/* Monitor the two quantities that the convergence analysis bounds (Sec. 4.2, assumptions "bounded gradients"
 * and "bounded staleness"): the squared norm of every applied worker delta and the squared distance between
 * the local model and the global model it is about to merge.  Computed inside the update and merge passes
 * (wavefront reductions, per-workgroup partial sums, one small reduction kernel); they never feed back into
 * the state.  Honoured at halos_gps_create; every LPS of that GPS then owns a small scratch buffer. */
#define HALOS_FLAG_NORMS 1u

/* Form the accumulated update the way Algorithm 1's LPS block writes it, Delta = theta_t - theta_{t_last}, instead of
 * keeping a running sum: the third buffer of every LPS then holds the snapshot theta_{t_last} (written by
 * halos_lps_create and by every merge), ordinary updates do not touch it (20 or 18 bytes per parameter instead of
 * 28 or 26), and the update that completes the accumulation overwrites it with theta_{t_last} - theta_t.  Same
 * quantity as the running sum, but rounded differently: the difference of two model-sized fp32 numbers carries an
 * absolute error of about one unit in the last place of the MODEL, i.e. a relative error near 1e-4 of a typical
 * accumulated update, against 1e-7 for the running sum.  Honoured at halos_gps_create. */
#define HALOS_FLAG_SNAPSHOT 2u

/* The global server keeps no momentum: beta_g = 0, the setting the paper uses for non-i.i.d. data (Sec. 5.4).  `M` of
 * halos_gps_create may be NULL and is never touched; a GPS update moves 16 bytes per parameter instead of 24 and gives
 * the model the general rule gives at beta = 0 (up to the sign of an exact zero).  global.beta must be 0 and stay 0;
 * halos_gps_push_update and a momentum delay are refused (ESTATE).  Honoured at halos_gps_create. */
#define HALOS_FLAG_GPS_NO_MOMENTUM 4u

/* Merges do not clear the third buffer (12 bytes per parameter instead of 16): the returned global model stays there
 * and the first update that accumulates afterwards overwrites it with 0 + its step instead of adding to it (4 bytes
 * less, once per accumulation).  Every result is the same, bit for bit; only the buffer's contents between a merge
 * and the next update are unspecified (logically zero).  Not with HALOS_FLAG_SNAPSHOT.  Honoured at halos_gps_create. */
#define HALOS_FLAG_DEFER_CLEAR 8u

/* Momentum kept in bfloat16, at both tiers: the M tensors of halos_gps_create and the m tensors of every
 * halos_lps_create are arrays of numel 16-bit elements (half the bytes; same 16-byte alignment).  After
 * m <- beta m + g the new momentum is rounded to bfloat16 (round to nearest, ties to even, decided on the fp32 value;
 * a NaN becomes 0x7FC0), and it is the rounded value that enters the step and is stored; models, accumulated updates
 * and returned global models stay fp32.  An option of this library, not of the paper (which does not state the
 * servers' precision; its workers train in fp16, Sec. 5.1): 4 bytes per parameter less on every update (LPS and GPS),
 * results that differ from the fp32-momentum run by the rounding.  Not available with a momentum delay above 1
 * (ESTATE).  Honoured at halos_gps_create. */
#define HALOS_FLAG_BF16_MOMENTUM 16u

/* What one halos_lps_step did. */
typedef struct {
    int32_t kind;         /* 0 queue was empty, 1 applied a worker delta, 2 merged a global model */
    int32_t delta_ready;  /* 1 if this update reached the accumulation count: the accumulated
                             update is now frozen and waits for halos_gps_merge               */
    int32_t accumulated;  /* 1 if this update was added to the accumulated update             */
    int32_t worker;       /* worker whose delta was applied, -1 otherwise                     */
    int64_t t;            /* number of worker updates applied so far (Alg. 1, LPS counter t)  */
    int64_t t_last;       /* value of t at the last merge (Alg. 1, LPS merge step)            */
} halos_step_info;

/* Protocol phase of an LPS with respect to its accumulated update. */
enum {
    HALOS_PHASE_ACCUMULATING = 0,  /* collecting updates; nothing in flight         */
    HALOS_PHASE_SENT = 1,          /* frozen update waits for halos_gps_merge       */
    HALOS_PHASE_RETURNING = 2,     /* GPS applied it; global model not yet arrived  */
    HALOS_PHASE_QUEUED = 3         /* global model sits in the LPS queue            */
};

/*
 * Create the GPS (Algorithm 1, REQUIRE line and GPS block).
 *   layout   tensor list (copied).  Tensors with numel 0 are allowed and skipped.
 *   hp       hyper-parameters (copied); hp->global is the GPS rule.
 *   Theta    device tensors holding the initial model Theta_0 (read and later updated in place).
 *   M        device tensors for the GPS momentum; zero-filled on `stream` by this call (NULL under HALOS_FLAG_GPS_NO_MOMENTUM;
 *            16-bit elements under HALOS_FLAG_BF16_MOMENTUM).
 * Errors: EINVAL (null/misaligned pointers, n_tensors < 1, negative numel, more than 2^32-1 elements
 * in one tensor, non-finite or out-of-range hyper-parameters), ENOMEM, EHIP.
 */
halos_status halos_gps_create(const halos_layout *layout, const halos_hparams *hp,
                              void *const *Theta, void *const *M, void *stream, halos_gps **out);

/*
 * Create one LPS attached to `gps` (Algorithm 1, LPS initialisation: theta_0 <- Theta_0, t <- 0, t_last <- 0).
 *   lps_id      caller's label for this server, >= 0 (reported in error strings only)
 *   n_workers   number of workers that may push to it, >= 1
 *   theta,m,acc device tensors of the layout.  On `stream` this call copies the GPS's CURRENT model into
 *               theta and zero-fills m and acc (under HALOS_FLAG_SNAPSHOT acc receives the model too; under
 *               HALOS_FLAG_BF16_MOMENTUM m has 16-bit elements).  `acc` is the server's third buffer: it holds the
 *               accumulated update G = theta_{t_last} - theta_t while collecting, stays frozen while that
 *               update is in flight, is overwritten with the returned global model by halos_gps_merge,
 *               and is zeroed again by the merge step.
 * The LPS keeps a pointer to the GPS (see the destroy calls for the order in which handles may go).
 */
halos_status halos_lps_create(halos_gps *gps, int32_t lps_id, int32_t n_workers,
                              void *const *theta, void *const *m, void *const *acc,
                              void *stream, halos_lps **out);

/*
 * A worker's delta arrives (Algorithm 1, LPS block: "receive delta").  Appends it to the LPS queue (Sec. 4.1 item 2); no device work.
 *   worker     0 <= worker < n_workers; a worker may have only one delta queued at a time (else ESTATE)
 *   g          device tensors of the layout holding the pseudo-gradient, dtype fp32 or bf16; borrowed
 *              until the halos_lps_step that applies it has finished on its stream
 *   staleness  number of server updates since the worker pulled its start model; carried as metadata
 *              (HALoS applies no staleness scaling) and readable through halos_lps_get_counters
 */
halos_status halos_lps_push_update(halos_lps *lps, int32_t worker, const void *const *g,
                                   halos_dtype dtype, uint32_t staleness);

/*
 * The same arrival with a scalar weight on the delta: the server applies ModelUpdate to weight * g (one fp32 product per
 * element inside the pass; weight = 1 is halos_lps_push_update exactly).  This is the hook for staleness-scaled
 * updates, the rule of the asynchronous-federated baseline in the paper's ablation (Sec. 5.2); the paper names only the
 * exponent of that method's polynomial, so the weight's formula is the caller's.  HALoS itself uses weight 1.
 *   weight   finite (EINVAL otherwise); the |g|^2 monitor sees the weighted delta
 */
halos_status halos_lps_push_update_weighted(halos_lps *lps, int32_t worker, const void *const *g, halos_dtype dtype,
                                            uint32_t staleness, float weight);

/*
 * The same arrival with the worker's END model theta_{t,H} in place of its delta: the subtraction of Algorithm 1's
 * worker block (delta = theta_{t,H} - theta_{t,0}) moves from the worker into the server's update pass, which forms the
 * pseudo-gradient g = theta_{t,0} - theta_{t,H} per element in fp32 -- the value a worker computing it in fp32
 * would have sent -- and then proceeds exactly as for halos_lps_push_update.  theta_{t,0} is read from the buffer
 * registered for the worker with halos_lps_set_worker_model: the model the server wrote there when the worker last
 * pulled, which the worker must have left unchanged (it trains in `end_model`).  The update must be applied with
 * halos_lps_step_pull, whose pass replaces theta_{t,0} by the new model right after reading it; halos_lps_step on
 * such an item is ESTATE.  The worker saves its subtraction pass and the delta buffer; the server reads 4 more
 * bytes per parameter than for an fp32 delta.
 *   end_model  device tensors of the layout, fp32, 16-byte aligned; borrowed like `g` above
 * ESTATE if the worker has no registered model buffer or already has an item queued; EINVAL if a tensor of `end_model`
 * overlaps the worker's registered model buffer (the start model would be read from what the worker trained in);
 * otherwise as halos_lps_push_update.
 * The |g|^2 monitor, where enabled, sees the g formed here.
 */
halos_status halos_lps_push_end_model(halos_lps *lps, int32_t worker, const void *const *end_model, uint32_t staleness);

/*
 * The global model sent back by the GPS arrives (Algorithm 1, LPS block: "receive Theta_i").  Appends it to the same queue as
 * the worker deltas; no device work.  ESTATE unless a halos_gps_merge for this LPS has run and its
 * result has not been delivered yet.
 */
halos_status halos_lps_push_global(halos_lps *lps);

/*
 * Handle the head of the LPS queue, in arrival order (Sec. 4.1 item 2).
 *   worker delta (the update branch of the LPS block): t <- t+1; one fused pass applies ModelUpdate(theta, g, eta_l, beta_l) and,
 *       unless an accumulated update is in flight, adds the applied step to acc.  If t - t_last has reached
 *       K and nothing is in flight, acc is frozen as the outgoing update (delta_ready = 1).
 *   global model (the merge branch of the LPS block): t_last <- t; theta <- (1-alpha) theta + alpha Theta_i; acc <- 0.
 * An empty queue is not an error (kind = 0).  `info` may be NULL.
 */
halos_status halos_lps_step(halos_lps *lps, void *stream, halos_step_info *info);

/*
 * Register the device tensors in which worker `worker` keeps the model it starts a round from, so that
 * halos_lps_step_pull can hand the updated model back in the same pass that applies the worker's delta.
 * The pointers are written into the server's device table by a small kernel on `stream`, i.e. in stream order:
 * steps issued before this call keep using the old buffers, steps issued after it (on `stream`, or on a stream
 * ordered after it) use the new ones.  No synchronisation.  The buffers are borrowed for the life of the handle
 * (or until re-registered).
 */
halos_status halos_lps_set_worker_model(halos_lps *lps, int32_t worker, void *const *model, void *stream);

/*
 * halos_lps_step with "Schedule the worker theta_t" (Algorithm 1, LPS block) fused in: if the head of the
 * queue is a worker delta, the pass that applies it also writes the updated model theta_t into that
 * worker's registered model buffer -- one read-modify-write pass instead of an update pass plus a copy
 * (halos_pull_model).  Results are identical to halos_lps_step followed by halos_pull_model.  If the head
 * is a global model the call behaves exactly like halos_lps_step.
 * ESTATE if the worker at the head has no registered model buffer (nothing is modified).
 */
halos_status halos_lps_step_pull(halos_lps *lps, void *stream, halos_step_info *info);

/*
 * Averaged step: the `count` (1..4) worker deltas at the head of the queue are averaged -- (w_1 g_1 + ... + w_n g_n) / n,
 * added in arrival order, the 1/n formed in fp32 -- and applied as ONE update of Algorithm 1's LPS block (t advances by
 * one; the accumulated update and the send test see one update).  This is the synchronous outer step of the
 * Local-SGD methods the paper compares with (Sec. 2: average the workers' deltas, then one momentum step), in one pass:
 * n deltas are read, the server's state is read and written once.  count = 1 is halos_lps_step.
 * ESTATE (nothing modified) unless the first `count` items are worker deltas of one element type, none of them an end
 * model; also under a momentum delay or HALOS_FLAG_NORMS.  Workers read the new model with halos_pull_model.
 * info->worker is the last of the averaged senders.
 */
halos_status halos_lps_step_average(halos_lps *lps, int32_t count, void *stream, halos_step_info *info);

/*
 * Batched steps: if several worker deltas wait at the head of the queue, apply up to max_items (1..4) of them in ONE
 * pass, one after the other in arrival order while each element is in registers.  Results -- state, counters, the
 * accumulated update, the send test, the models handed back -- are those of that many single steps, bit for bit; only
 * m, theta and the third buffer are read and written once instead of once per delta (k deltas: 2k + 28 + 4k bytes per
 * parameter instead of 30k, bf16 deltas with the model handed back).  The queue sentence of Sec. 4.1 is respected: a
 * batch never reaches past a queued global model.  If a returned global model is AT the head and worker deltas wait
 * right behind it, the pass opens with the merge (Algorithm 1's merge branch, then the updates, on each element while
 * it is in registers): the same results as halos_lps_step followed by the updates, without the merge's own pass over
 * the model and the third buffer (16 bytes per parameter less).  Such a batch is the merge plus up to max_items - 1
 * deltas, and is taken already when one delta waits.  Under a momentum delay the merge and ONE delta behind it share a
 * pass (with pull non-zero); more deltas do not.
 *   pull      non-zero: each update also writes the model right after it to its sender's registered buffer
 *             (halos_lps_step_pull for every item)
 *   infos     host array of max_items entries; entry i describes the i-th step taken
 *   n_done    number of queue items handled: 0 (empty queue), 1 (a merge with no delta behind it, or a single update:
 *             whenever fewer than two items can share a pass, or the server runs a momentum delay or the norm
 *             monitors, the call is exactly halos_lps_step / halos_lps_step_pull), or the size of the batch
 * Errors as for halos_lps_step_pull; nothing is modified on error.
 */
halos_status halos_lps_step_batch(halos_lps *lps, int32_t max_items, int32_t pull, void *stream, halos_step_info *infos,
                                  int32_t *n_done);

/*
 * The accumulated update of LPS `from` reaches the GPS (Algorithm 1, GPS block): one fused pass applies
 * ModelUpdate(Theta, G, eta_g, beta_g) and writes the new global model Theta_i over `from`'s third buffer,
 * where it stays frozen until `from` merges it -- later GPS updates do not change it.
 * ESTATE unless `from` has a frozen update waiting (delta_ready was reported and not yet consumed).
 */
halos_status halos_gps_merge(halos_gps *gps, halos_lps *from, void *stream);

/*
 * Single tier: the global server applies a worker's delta itself, Theta <- ModelUpdate(Theta, weight * g, eta_g, beta_g),
 * with its own momentum (and its delayed-momentum cycle, if one is set): the server of the single-level asynchronous
 * baseline that the paper compares with (Sec. 2; App. D lists its hyper-parameters).  One fused pass, 20 bytes per
 * parameter for an fp32 delta (18 for a 16-bit one); nothing is sent back -- workers read the model with
 * halos_pull_model.  Counts as one update of the GPS.  Local servers attached to the same GPS are unaffected.
 *   g, dtype   as for halos_lps_push_update; borrowed until the pass has finished on `stream`
 * ESTATE under HALOS_FLAG_GPS_NO_MOMENTUM; EINVAL as for halos_lps_push_update.
 */
halos_status halos_gps_push_update(halos_gps *gps, const void *const *g, halos_dtype dtype, float weight, void *stream);

/*
 * Copy a server's current model into caller tensors ("Schedule the worker theta_t" in Algorithm 1's LPS block; also
 * usable to read the global model).  server is a halos_lps* (is_gps = 0) or a halos_gps* (is_gps = 1).
 * dst: device tensors of the layout, fp32.
 */
halos_status halos_pull_model(const void *server, int32_t is_gps, void *const *dst, void *stream);

/*
 * Replace hyper-parameters between events (learning-rate schedules belong to the caller; the theorem of
 * Sec. 4.2 allows a time-varying rate).  For an LPS: hp->local, hp->alpha and hp->K take effect from the
 * next step.  For the GPS: hp->global.  Other fields are validated but ignored.
 */
halos_status halos_set_hparams(void *server, int32_t is_gps, const halos_hparams *hp);

/* Drop what a server remembers about pointer sets it has already checked (deltas per worker, pull destinations, the
 * norm output; for the GPS: deltas of halos_gps_push_update): the next use of any pointer set is checked again.
 * For callers that free buffers and may get the same addresses back for smaller allocations. */
halos_status halos_forget_buffers(void *server, int32_t is_gps);

/* Change only the accumulation count K of one LPS (>= 1), effective from the next step. */
halos_status halos_lps_set_threshold(halos_lps *lps, int32_t K);

/*
 * Read the protocol counters of an LPS.  Any out pointer may be NULL.
 *   t, t_last     as in Algorithm 1
 *   phase         one of HALOS_PHASE_*
 *   queued        items waiting in the queue
 *   max_staleness largest staleness value seen in halos_lps_push_update
 */
halos_status halos_lps_get_counters(const halos_lps *lps, int64_t *t, int64_t *t_last, int32_t *phase,
                                    int32_t *queued, uint32_t *max_staleness);

/*
 * Read the monitors of an LPS created under HALOS_FLAG_NORMS: out[0] = sum of g^2 over all parameters for the
 * most recent worker update, out[1] = sum of (theta - Theta_i)^2 just before the most recent merge (0 until the
 * first one).  `out` is a host array of two doubles.  The call waits for `stream`.
 * ESTATE if the flag was not set when the GPS was created.
 */
halos_status halos_lps_get_norms(const halos_lps *lps, void *stream, double *out);

/*
 * halos_lps_step for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid it) and still want the monitors of HALOS_FLAG_NORMS: works on ANY local server, with
 * or without that flag, and never calls hipMalloc / hipFree.  The per-workgroup partial sums go to a fixed array in
 * the library's device image (one copy per GPU, 16384 doubles = 128 KiB, held until the process ends) instead of a
 * buffer owned by the server.
 *   norms_out  device pointer, 8-byte aligned, to two doubles owned by the caller: a step that applies a worker
 *              delta writes the sum of g^2 to norms_out[0], a step that merges a global model writes the sum of
 *              (theta - Theta_i)^2 before the merge to norms_out[1]; the other element is left as it is, and an empty
 *              queue writes nothing.  Written on `stream`; same values, bit for bit, as halos_lps_get_norms reports
 *              after halos_lps_step on a server created under the flag.
 * Everything else (state, counters, `info`, errors) is exactly halos_lps_step.  The server's own monitors, if it has
 * any, are not updated by this call.
 * Limit: one partial sum per workgroup per launch, i.e. blocks_per_cu x compute units per 384 tensors of the
 * layout; EINVAL (nothing modified) if that exceeds 16384.  With the default launch shape (one workgroup per compute
 * unit) a layout of up to 24,576 tensors fits on a 256-unit device.
 * Every call on a GPU shares that GPU's array: calls that may run concurrently on one GPU (different streams, different
 * servers) race on it and give wrong NORMS (state is unaffected); issue them on one stream or order the streams.
 */
halos_status halos_lps_step_norms(halos_lps *lps, void *stream, halos_step_info *info, double *norms_out);

/* Number of accumulated updates the GPS has applied (the index i of Algorithm 1's GPS loop). */
halos_status halos_gps_get_counters(const halos_gps *gps, int64_t *updates);

/*
 * Delayed Nesterov momentum at a server (the optimizer of the paper's runs at both tiers: Sec. 5.1; the
 * hyper-parameter table of App. D lists the delays d_l, d_g and gives the rates it prints as
 * eta / d).  The paper takes the rule from the Async-Local-SGD work it cites; with
 * that work's default of no momentum between refreshes, and this paper's coefficient cg on the gradient
 * term, a server with rule (eta, beta, cg) and delay d handles its updates in cycles of d:
 *     every update:            buffer <- buffer + g;   x <- x - eta * (cg / d) * g
 *     the d-th of a cycle:     m <- beta * m + buffer / d;   x <- x - eta * [ (cg / d) * g + beta * m ];
 *                              buffer <- 0
 * (x is theta_l with g a worker's pseudo-gradient, or Theta with g the accumulated update G.)  d = 1 is
 * ModelUpdate of App. E, the rule the servers start with.  The accumulated update, the threshold K, the
 * merge and the pull are unchanged; a merge does not touch the buffer or the position in the cycle.
 *
 *   d       delay, >= 1.  d = 1 switches back to the plain rule; `buffer` is then ignored and may be NULL.
 *   buffer  for d > 1: device tensors of the layout, fp32, 16-byte aligned, borrowed for the life of the handle
 *           (or until replaced).  They need no initialisation: the first update of a cycle overwrites them,
 *           and between a refresh and the next update their contents are unspecified (logically zero).
 *
 * fp32 operation order per element (1/d and cg * (1/d) are formed once, in fp32, on the host):
 *     b1 = b + g  (b1 = g for the first update of a cycle);  gp = (cg/d) * g;
 *     plain update:  s = eta * gp;                          refresh:  m1 = fma(beta, m, b1 * (1/d));
 *                                                                     s = eta * fma(beta, m1, gp);
 *     x = x - s;  accumulated update as in halos_lps_step.
 * Updates that do not refresh never read or write the momentum, so they move as many bytes as a plain update.
 *
 * The call writes the pointers into the server's device table in stream order on `stream` (no synchronisation;
 * see halos_lps_set_worker_model).  Allowed only between cycles (before the first update, or when the last update was a refresh):
 * ESTATE otherwise.  EINVAL for d < 1, or a bad `buffer` with d > 1.  The delayed kernels always use
 * non-temporal accesses (halos_set_launch_config's `nontemporal` does not apply to them).
 */
halos_status halos_lps_set_momentum_delay(halos_lps *lps, int32_t d, void *const *buffer, void *stream);
halos_status halos_gps_set_momentum_delay(halos_gps *gps, int32_t d, void *const *buffer, void *stream);

/* The delay d of a server and the number of updates applied since its last refresh (0 .. d-1).  Either may be NULL. */
halos_status halos_lps_get_momentum_delay(const halos_lps *lps, int32_t *d, int32_t *seen);
halos_status halos_gps_get_momentum_delay(const halos_gps *gps, int32_t *d, int32_t *seen);

/*
 * Launch shape for all later kernel launches of the calling process.
 *   blocks_per_cu  persistent workgroups per compute unit, 1..64 (0 = keep; the library starts with 1)
 *   nontemporal    1 = stream state through the caches with non-temporal accesses, 0 = plain, -1 = keep
 * Returns EINVAL for out-of-range values.
 */
halos_status halos_set_launch_config(int32_t blocks_per_cu, int32_t nontemporal);

/*
 * Device memory sorted by HBM region (a set-up helper, not a step of the algorithm; the one place where this library
 * owns parameter-sized memory).  An MI355X serves its HBM from a few large regions, handed to a process one after
 * the other, and an update pass whose arrays lie in different regions runs about a fifth faster than one whose
 * arrays share a region (halos_probe.h has the measurement call this is built on).  The arena allocates 2 GiB slabs
 * until it holds, for every placement class, enough slabs from a region of its own, sorts them by timing each new
 * slab against one slab per region found so far, and releases what it does not need.  Classes are the caller's:
 * arrays that one pass touches together should go to different classes.  The benchmark uses three: {momenta, third
 * buffers}, {local models, deltas, GPS momentum}, {worker model buffers, GPS model}.
 *   n_classes        1..8
 *   bytes_per_class  host array: bytes the caller will ask for in each class
 *   max_walk_bytes   upper bound on the memory held DURING the search (0 = all free memory but 8 GiB).  Memory is
 *                    handed out in region order, so reaching the third region means holding the first two: on an
 *                    otherwise idle 288 GB device the search holds up to ~230 GiB for a few seconds.
 * If fewer regions than classes are found (other processes hold memory, a smaller device, a low bound) classes share
 * regions: slower, still correct.  Errors: EINVAL, ENOMEM, EHIP (from the timing kernel).
 * The calling thread's current device is used; the search runs on the default stream and waits for it.
 */
typedef struct halos_arena halos_arena;
halos_status halos_arena_create(int32_t n_classes, const uint64_t *bytes_per_class, uint64_t max_walk_bytes,
                                halos_arena **out);

/* Hand out `bytes` (> 0) of device memory from the slabs of class `cls`, 256-byte aligned, uninitialised; it stays
 * valid until halos_arena_destroy.  An allocation never straddles two slabs.  When a class has used up its region's
 * slabs, further slabs come from wherever the device has memory left (placement unknown); a request larger than a
 * slab (2 GiB) gets an allocation of its own, likewise.  ENOMEM when the device is full. */
halos_status halos_arena_alloc(halos_arena *arena, int32_t cls, uint64_t bytes, void **ptr);

/* What the search found.  Any out pointer may be NULL; region_of_class and slabs_of_class are host arrays of
 * n_classes entries (region index of each class, -1 if none; slabs it currently holds). */
halos_status halos_arena_info(const halos_arena *arena, int32_t *n_regions, uint64_t *walked_bytes,
                              double *same_region_gbps, int32_t *region_of_class, int32_t *slabs_of_class);

/* Wait for the device, then free every slab.  Pointers handed out by the arena die with it.  NULL is ignored. */
void halos_arena_destroy(halos_arena *arena);

/* Release the handle's tables (this waits for the device: work that still uses them finishes first).
 * Caller buffers are untouched.  NULL is ignored.  A GPS destroyed while local servers are still attached to it
 * must not be used again, but its layout tables, which those servers launch with, stay alive until the last of
 * them is destroyed: the order of the destroy calls does not matter. */
void halos_lps_destroy(halos_lps *lps);
void halos_gps_destroy(halos_gps *gps);

/* Description of the calling thread's most recent error ("" if none). */
const char *halos_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HALOS_H */
