/*
 * asyncmesh.h -- C ABI of the MI355X (gfx950) implementation of the AsyncMesh per-stage update.
 *
 * One pipeline stage of n parameters is replicated R times (R = m, the number of data-parallel
 * replicas in the paper's 2D mesh).  Every training step each replica
 *   (1) takes its local optimizer step        w^_i^t = OPT(w_i^{t-1}, g_i^{t-1})
 *                                             [sparse-averaging equation, first line],
 *   (2) sends w^_i^t[S^t], a random subset of its coordinates, towards the other replicas
 *                                             [Sec. "Asynchronous sparse averaging"],
 *   (3) receives the average that was sent tau averaging rounds ago and applies it with the
 *       EMA-of-staleness correction           [Sec. "Delay correction via estimating average
 *                                              staleness": the EMA and estimated-average equations
 *                                              and the corrected update that follows them],
 *   (4) extrapolates the optimizer's displacement to get the weights of the next forward pass
 *                                             [Sec. "Asynchronous pipeline parallelism": NAG-style
 *                                              look-ahead of the last update direction].
 * The R replicas and the delay buffer (appendix, wall-clock paragraph: the asynchronous set-up is
 * simulated with a buffer of delayed copies) live side by side in the memory of ONE GPU.
 *
 * General conventions
 *   - Every pointer marked DEVICE is memory of the GPU that was current at am_init_state; it is
 *     owned by the caller, must stay valid until am_destroy, and must be 16-byte aligned
 *     (bf16 arrays: 8-byte aligned).  Pointers marked HOST are ordinary host memory, read during
 *     the call only.
 *   - All work is enqueued on the stream given to am_init_state (am_lookahead: its own argument).
 *     No call synchronises with the device, allocates device memory, or copies to the host,
 *     except am_read_flags and am_get_profile, which say so.
 *   - Every function returns AM_OK (0) or a negative am_status.  On an error the state (host
 *     record and the caller's arrays) is unchanged and the call may be repeated; argument errors
 *     are found before anything is enqueued (a step whose kernel launch itself fails may already
 *     have enqueued its subset-offsets pass, which a repeated call simply redoes).
 *     am_last_error() gives a message for the calling thread.
 *   - No exception crosses this boundary.
 */
#ifndef ASYNCMESH_H
#define ASYNCMESH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AM_MAX_REPLICAS 32u

typedef struct am_state am_state;      /* opaque, host side, owned by the library */

typedef enum {
    AM_OK      =  0,
    AM_EINVAL  = -1,    /* bad argument or configuration                                   */
    AM_EALIGN  = -2,    /* a device pointer is not aligned as required                     */
    AM_ENOMEM  = -3,    /* workspace too small / host allocation failed                    */
    AM_EORDER  = -4,    /* step index is not the previous one plus one                     */
    AM_EHIP    = -5,    /* a HIP runtime call failed (message has the HIP error string)    */
    AM_EOVERFLOW = -6   /* am_read_flags has reported a subset that did not fit its ring slot:
                           the state no longer follows the method, further steps are refused  */
} am_status;

/* local optimizer (experimental-setup appendix: NAdamW with momentum 0.99 for asynchronous
 * pipelines, AdamW for synchronous ones; SGD is what the equations are written for)         */
typedef enum {
    AM_OPT_SGD    = 0,  /* m <- beta1 m + g ; w^ = w (1 - lr wd) - lr m   (beta1 = 0: plain SGD, m untouched) */
    AM_OPT_ADAMW  = 1,  /* Adam moments, bias correction, decoupled weight decay              */
    AM_OPT_NADAMW = 2   /* Adam with Nesterov momentum (Dozat's schedule), decoupled decay    */
} am_opt;

typedef enum {
    AM_CORR_NONE  = 0,  /* subset <- old average                 (asynchronous sparse averaging equation) */
    AM_CORR_EMA   = 1,  /* subset <- old average + EMA of staleness   (EMA equation + corrected update)    */
    AM_CORR_EAGER = 2   /* subset <- old average + (1/m)(w^_i^t - w^_i^{t-tau}), no memory: the eager-DiLoCo
                           special case named at the end of the delay-correction section (with p = 1)      */
} am_corr;

typedef enum { AM_F32 = 0, AM_BF16 = 1 } am_dtype;

/* Precision of the values put on the wire (the paper's compression experiment: quantising the
 * exchanged subset).  The old average is formed from the quantised values (accumulated exactly,
 * rounded to fp32); a replica's own staleness term uses its own exact old value. */
typedef enum {
    AM_MSG_F32  = 0,
    AM_MSG_BF16 = 1,    /* round to nearest even                                                     */
    AM_MSG_E4M3 = 2     /* 8-bit float 1-4-3, bias 7, no infinity, max 448; nearest even, saturating */
} am_msg;

/* How the subset S^t is drawn.  BERNOULLI is the paper's sampling model (Section 3.2; the
 * sparse-averaging lemma of the appendix: every element in the subset with probability p,
 * independently).  STRATIFIED is a VARIANT with an exact subset size: the coordinates are cut into
 * aligned blocks of B = round(1/p) and exactly one coordinate of every block is in S^t, at offset
 * floor(X_b B / 2^32), X_b the generator word that coordinate number b = mu / B would get in the
 * Bernoulli scheme.  Every coordinate is in S^t with probability 1/B (the marginal the lemma's
 * proof uses), |S^t| = n / B up to the cut last block, and no ring slot can overflow. */
typedef enum {
    AM_SUBSET_BERNOULLI  = 0,
    AM_SUBSET_STRATIFIED = 1
} am_subset;

/* How the EMA vectors d_i lie in memory.  S^t is the same for every replica (Sec. "Sparse parameter
 * averaging"), so the entries of d that one step touches are the same coordinates in every replica.
 *   PER_REPLICA: one flat array of n floats per replica (what a replica on its own GPU would hold).
 *   INTERLEAVED: the replicas are cut into blocks of rb = min(8, R rounded up to a power of two)
 *     consecutive replicas; a block is ONE array [coordinate][replica in block] of
 *     ceil(n / 256) * 256 * rb floats (whole tiles; entries of absent replicas and of coordinates
 *     >= n are never changed).  A 128-byte line then holds 32 / rb coordinates of all the block's
 *     replicas, so far fewer lines are touched per step (R = 8, p = 5 %: 18.5 % of the lines
 *     instead of 80.6 %).  A property of holding all replicas on one GPU.  am_d_layout_info gives rb,
 *     the number of blocks and the floats per block. */
typedef enum {
    AM_D_PER_REPLICA = 0,
    AM_D_INTERLEAVED = 1
} am_dlayout;

typedef struct {
    uint64_t n;              /* d_j: parameters of the stage, per replica; 1 <= n < 2^32 - 2^20          */
    uint32_t replicas;       /* m = R, 1 .. AM_MAX_REPLICAS                                              */
    uint32_t delay;          /* tau >= 0, counted in averaging rounds (tau*K steps)                      */
    uint32_t avg_interval;   /* K >= 1: averaging happens at steps t with t mod K == 0                   */
    uint32_t optimizer;      /* am_opt                                                                   */
    double   fraction;       /* p in (0, 1]: every coordinate is in S^t independently with probability p */
    uint64_t seed;           /* shared by all replicas of the stage; S^t is a pure function of (seed, t) */
    float    beta1, beta2, eps, weight_decay;
    float    gamma;          /* look-ahead coefficient (used when lookahead != 0)                        */
    uint32_t lookahead;      /* 0: fwd = w ; 1: fwd = w + gamma (w^ - w_before_step)                     */
    uint32_t correction;     /* am_corr                                                                  */
    uint32_t fwd_dtype;      /* am_dtype of the fwd arrays                                               */
    uint32_t grad_dtype;     /* am_dtype of the gradient arrays                                          */
    double   momentum_decay; /* NADAMW only: psi of mu_t = beta1 (1 - 0.5 * 0.96^(t psi)); usual 0.004   */
    uint32_t subset_granule; /* 1 (or 0): coordinates drawn independently, the paper's sampling model.
                                32: VARIANT, not the paper's: aligned blocks of 32 coordinates (one
                                128-byte line) drawn as a whole, block b in place of coordinate b in
                                the generator; same inclusion probability p per coordinate.         */
    uint32_t msg_dtype;      /* am_msg: precision of the exchanged subset values                        */
    uint32_t subset_kind;    /* am_subset: how S^t is drawn                                             */
    uint32_t d_layout;       /* am_dlayout: memory layout of the EMA vectors                            */
    uint64_t ring_cap_lines; /* 0: a ring slot is sized from the distribution of |S^t| (see
                                am_workspace_bytes).  Else: the number of 128-byte lines per block a slot
                                gets, for callers that bound the workspace themselves; tiles that do
                                not fit are left out of that round's average and flag bit 0 is raised */
} am_config;

/* The subset: S^t = { mu in [0, n) : X(seed, t, mu) < floor(p * 2^32) }, X = word (mu & 3) of
 * Philox4x32-10 with counter (lo32(mu>>2), hi32(mu>>2), lo32(t), hi32(t)) and key (lo32(seed),
 * hi32(seed)).  This is the sampling model of the sparse-averaging lemma (each element in the
 * subset with probability p, independently). */

typedef struct {
    /* HOST arrays of `replicas` DEVICE pointers each; every pointed-to array has n elements.   */
    float *const *w;        /* master weights, fp32, in: w^{t-1}, out: w^t                       */
    float *const *m;        /* first moment / momentum, fp32 (may be NULL for SGD with beta1=0)  */
    float *const *v;        /* second moment, fp32 (may be NULL for SGD)                         */
    float *const *d;        /* EMA of staleness d_i, fp32 (may be NULL when correction = NONE);
                               d_layout = INTERLEAVED: one pointer per BLOCK instead (am_d_layout_info) */
    void  *const *fwd;      /* weights for the next forward pass, fwd_dtype; NULL = not produced
                               (allowed only with lookahead = 0 and fwd_dtype = AM_F32)          */
    void    *workspace;     /* DEVICE, 256-byte aligned: delay ring + subset offsets + flags     */
    uint64_t workspace_bytes;
} am_buffers;

/* Bytes of workspace a configuration needs.  The delay ring inside it holds tau+1 slots; a slot
 * keeps the replicas of a block (rb <= 8 consecutive replicas) side by side, [coordinate][replica]:
 * every tile of 256 coordinates owns, per block, ceil(X rb / 32) whole 128-byte lines, X its number
 * of selected coordinates; a slot has room for the expected number of lines plus twelve standard
 * deviations (stratified sampling: exactly what the fullest tile can need, times the tiles), or for
 * ring_cap_lines lines when the config names a size. */
am_status am_workspace_bytes(const am_config *cfg, uint64_t *out_bytes);

/* Shape of the EMA vectors under the config's d_layout: replicas per block (PER_REPLICA: 1), number
 * of arrays buffers.d must point to, and floats per array.  Any of the outputs may be NULL. */
am_status am_d_layout_info(const am_config *cfg, uint32_t *out_replicas_per_block, uint32_t *out_arrays,
                           uint64_t *out_floats_per_array);

/* Validate, bind the caller's buffers and the stream, and enqueue the zeroing of m, v, d (d^0 = 0,
 * experimental-setup appendix) and of the workspace.  w is left as given.  hip_stream is a
 * hipStream_t (NULL = the default stream).  The next step index is 1. */
am_status am_init_state(const am_config *cfg, const am_buffers *buf, void *hip_stream, am_state **out);

/* One fused step t (= previous t + 1): parts (1)-(4) above for all R replicas.
 *   grads      HOST array of R DEVICE pointers to n gradients each (grad_dtype), read only;
 *              reusable by the caller once the stream has passed this call.
 *   lr         eta for this step (the caller owns the schedule)
 *   lambda_t   EMA coefficient in [0, 1] for this step (the paper: 0.5, then cosine decay to 0.01)
 *   grad_scale gradients are multiplied by this first (e.g. a clipping factor); 1 = none */
am_status am_step(am_state *st, uint64_t t, const void *const *grads,
                  float lr, float lambda_t, float grad_scale);

/* am_step with one more gradient factor per replica, read from DEVICE memory (R floats) by the
 * kernel: g_i <- grad_scale * replica_scale[i] * g_i.  For global-norm clipping (norm 1 in the
 * paper's set-up) without a host round trip: am_grad_sqnorm gives the stage's share of each
 * replica's squared norm, the caller turns the norms of all stages into factors on the device. */
am_status am_step_scaled(am_state *st, uint64_t t, const void *const *grads, float lr, float lambda_t,
                         float grad_scale, const float *dev_replica_scale);

/* One tick of the heterogeneous set-up (Sec. "Heterogeneous setup" and its appendix paragraph:
 * devices of unequal speed; the averaging interval is proportional to the device speed, so faster
 * devices make more iterations between two averaging steps).  The R replicas advance in lock-step
 * ticks t = 1, 2, ...; replica i makes a local optimizer step in this tick iff bit i of
 * active_mask is set, with its own count of steps made so far in the bias corrections (and in
 * NADAMW's momentum schedule).  An idle replica keeps w, m, v (its w^ is its w, its look-ahead
 * displacement is zero) and grads[i] is not read (may be NULL); it still sends and receives when
 * the tick is an averaging step (t a multiple of avg_interval).  With every bit set in every tick
 * this is am_step_scaled.  am_step / am_step_scaled set every replica's count to t.
 * AM_EINVAL if a bit at or above `replicas` is set. */
am_status am_step_masked(am_state *st, uint64_t t, const void *const *grads, float lr, float lambda_t,
                         float grad_scale, const float *dev_replica_scale, uint32_t active_mask);


/* dev_out[i] (DEVICE, R doubles) = sum over the stage of g_i[mu]^2.  grads as for am_step.
 * Deterministic (fixed reduction order). */
am_status am_grad_sqnorm(am_state *st, const void *const *grads, double *dev_out);

/* Parts (2)-(3) alone, acting on the current w, which plays the role of w^ (for callers that run
 * their own optimizer).  Counts as step t.  m, v, fwd are not touched. */
am_status am_sparse_average(am_state *st, uint64_t t, float lambda_t);

/* Stateless part (4) in its literal two-point form: out = w + gamma (w - w_prev), n elements.
 * out (DEVICE, out_dtype) may alias neither input. */
am_status am_lookahead(void *out, uint32_t out_dtype, const float *w, const float *w_prev,
                       uint64_t n, float gamma, void *hip_stream);

/* The delay in force from the next step on: 0 <= tau <= the delay of the configuration (which sizes
 * the ring).  Models an average that arrives late or early (appendix: the asynchronous set-up is
 * simulated by buffering); a round may then be received twice or never.  Host value, no device work. */
am_status am_set_delay(am_state *st, uint32_t tau);

/* Diagnostics of the paper's consensus-error figure, enqueued on the stream, results in DEVICE
 * memory (3 doubles): out[0] = sum_i ||w_i - mean_i w_i||^2 (consensus error, appendix notation),
 * out[1] = mean and out[2] = max over the coordinates of the variance over the replicas of the EMA
 * estimates d_i (0 when there is no d).  Deterministic (fixed reduction order). */
am_status am_diagnostics(am_state *st, double *dev_out3);

/* Materialise S^t in ascending order: dev_out[0 .. count) (DEVICE, uint64, room for `capacity`
 * indices; more are dropped) and *dev_count = |S^t| (DEVICE, one uint64).  Any t >= 0. */
am_status am_subset_indices(am_state *st, uint64_t t, uint64_t *dev_out, uint64_t capacity,
                            uint64_t *dev_count);

/* am_subset_indices for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same result bit for bit, but the
 * per-tile offsets the three kernels share live in a static device array of the library
 * (2 MiB + 4.25 KiB, held by every GPU the library runs on until the process ends; its device
 * address is looked up once per device at am_init_state / am_resume_state) instead of the
 * caller's workspace, and the call allocates nothing, on the device or on the host.
 * Limit: n <= 2^27 = 134,217,728 coordinates; a larger stage is refused with AM_EINVAL (use
 * am_subset_indices).  The device that was current at am_init_state must be current (AM_EINVAL
 * otherwise).  Every call on one GPU uses that GPU's one array: calls that overlap on a GPU (two
 * states on different streams, two threads) race on it -- serialise them.  Nothing in the array has
 * to start at zero: every word a call reads it has written first. */
am_status am_subset_indices_static(am_state *st, uint64_t t, uint64_t *dev_out, uint64_t capacity,
                                   uint64_t *dev_count);

/* Synchronises the stream and returns sticky flags: bit 0 = some S^t needed more lines than a
 * ring slot holds (the tiles past the capacity were left out of that round's average, at send and
 * at receive alike; with the default slot size the chance is about 1e-33 per step).  Once this
 * call has reported bit 0, am_step* and am_sparse_average on the state return AM_EOVERFLOW. */
am_status am_read_flags(am_state *st, uint32_t *out_flags);

/* Optional timing of the fused step kernel alone: while on, am_step brackets that kernel with
 * events on its stream (at most 4096 launches between two am_get_profile calls; later ones run
 * untimed).  am_get_profile synchronises, returns the summed kernel time in milliseconds and the
 * number of launches timed since profiling was switched on (or since the last call), and resets
 * both.  am_get_profile_times additionally copies the individual launch times (milliseconds, in
 * launch order) to out_ms[0 .. min(launches, capacity)) before resetting. */
am_status am_set_profiling(am_state *st, int on);
am_status am_get_profile(am_state *st, double *out_kernel_ms, uint64_t *out_launches);
am_status am_get_profile_times(am_state *st, float *out_ms, uint64_t capacity, uint64_t *out_launches);

/* Slot capacity (fp32 positions per replica = lines * 32) and number of ring slots of this state;
 * host values, no device work. */
am_status am_ring_info(const am_state *st, uint64_t *out_capacity, uint32_t *out_slots);

/* Checkpoints.  Everything on the device is the caller's (w, m, v, d, fwd and the workspace, which
 * holds the delay ring of the appendix' "buffering" and the subset offset tables); what the library
 * itself remembers between steps is this small host record.  To checkpoint: let the stream drain,
 * copy the arrays and the workspace, call am_export_state.  To resume: put the bytes back (any
 * addresses, same alignment rules), and call am_resume_state instead of am_init_state; it clears
 * nothing.  S^t is a pure function of (seed, t), so there is no generator state to save.  The
 * record is refused (AM_EINVAL) when the config differs from the one it was exported under in a
 * field that shapes the ring, the subsets or the arrays (n, replicas, delay, avg_interval, optimizer,
 * fraction, seed, subset_granule, subset_kind, d_layout, ring_cap_lines).  Host-only calls apart
 * from what am_init_state does. */
typedef struct {
    uint64_t magic;             /* layout version of this record                                */
    uint64_t config_digest;
    uint64_t last_t;            /* the last step made                                           */
    uint64_t next_lines_step;   /* the step whose send subset is already sized in the workspace */
    uint32_t delay_now;         /* the delay in force (am_set_delay)                            */
    uint32_t reserved;
    uint64_t opt_steps[AM_MAX_REPLICAS];   /* optimizer steps each replica has made             */
    double   mu_product[AM_MAX_REPLICAS];  /* NADAMW: running product of the momentum schedule  */
} am_snapshot;

am_status am_export_state(const am_state *st, am_snapshot *out);
am_status am_resume_state(const am_config *cfg, const am_buffers *buf, void *hip_stream,
                          const am_snapshot *snapshot, am_state **out);

am_status am_destroy(am_state *st);

const char *am_last_error(void);      /* message of the last failing call on this thread */
const char *am_version(void);          /* "asyncmesh-gfx950 <version> src:<hash>": the hash is a digest of the
                                          library's source files taken when it was built */

#ifdef __cplusplus
}
#endif
#endif /* ASYNCMESH_H */
