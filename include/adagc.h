/*
 * libadagc — fused AdaGC + AdamW / Lion optimizer step for AMD gfx950 (MI355X).
 *
 * AdaGC (arxiv 2502.11034) clips every parameter tensor's gradient against an
 * exponential moving average of that tensor's own past (clipped) gradient
 * norms, before the gradient enters the optimizer's moments (Sec. 4.2, Eq. 3;
 * Alg. 1 in the appendix "Pseudocode of AdamW with AdaGC").  One call of
 * adagc_step performs, for a whole ragged list of parameter tensors:
 *
 *   1. n_i = ||g_i||_2 for every tensor i                      (Sec. 4.1 notation; Eq. 3)
 *   2. warm-up steps (t <= T_start): one global coefficient
 *        h = min{lambda_abs / ||g||, 1}                         (Eq. 2, Alg. 1)
 *        gamma_i = min{gamma_i, h*n_i}  (gamma_i = h*n_i on step 1)
 *      other steps: h_i = min{lambda_rel*gamma_i / n_i, 1},
 *        gamma_i = beta*gamma_i + (1-beta)*||h_i g_i||          (Eq. 3, Alg. 1)
 *   3. AdamW with the clipped gradient h_i*g_i                  (Alg. 1)
 *      or Lion with the clipped gradient (rule of Chen et al., which the paper
 *      cites but does not print).
 *
 * Conventions
 *   - Plain C ABI.  Every pointer is marked HOST or DEVICE below.  Device
 *     pointers belong to the GPU that was current when adagc_create ran.
 *   - All tensor storage (params, grads, moments, bf16 copies, ema_norms) is
 *     owned by the caller; the library never allocates or frees it.  The
 *     context owns only its segment table, reduction scratch and per-tensor
 *     result arrays.
 *   - Every function returns ADAGC_OK (0) or a negative error code; nothing
 *     throws or aborts.  Arguments are validated before any work is enqueued,
 *     so a failed call leaves all state untouched.
 *   - A context is not thread-safe; use one per host thread or lock around it.
 *   - All steps of one context share its pointer table, reduction scratch and
 *     result arrays on the GPU, so they must execute one after another: issue
 *     them on one stream, or order the streams yourself (an event between a
 *     step on stream A and the next step or adagc_get_* call on stream B).
 *     Steps of different contexts may overlap freely.
 */
#ifndef ADAGC_H
#define ADAGC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADAGC_OK                   0
#define ADAGC_ERR_INVALID_ARG     (-1)  /* NULL pointer, non-positive size, bad enum, bad hyper-parameter */
#define ADAGC_ERR_OOM             (-2)  /* host or device allocation failed */
#define ADAGC_ERR_HIP             (-3)  /* a HIP runtime call failed (no device, launch error, ...) */
#define ADAGC_ERR_TOO_LARGE       (-4)  /* the list needs more than 2^32-1 chunks, or has more than 2^24-1 tensors */
#define ADAGC_ERR_STATE           (-5)  /* call made in the wrong state (e.g. bf16 copies not set) */

#define ADAGC_OPT_ADAMW 0
#define ADAGC_OPT_LION  1
#define ADAGC_OPT_MUON  2   /* every tensor is a matrix; stepped with adagc_muon_step after adagc_muon_attach */
#define ADAGC_GRAD_F32  0
#define ADAGC_GRAD_BF16 1

/* Which clipping rule adagc_step applies (adagc_hyper.clip_mode). */
#define ADAGC_MODE_ADAGC         0  /* Alg. 1: GlobalGC warm-up for t_start steps, then per-tensor Eq. 3 */
#define ADAGC_MODE_GLOBALGC      1  /* Eq. 2 on every step (the paper's baseline); keeps no state */
#define ADAGC_MODE_GLOBAL_ADAGC  2  /* one adaptive threshold for the whole model (ablation "adaptive but
                                       non-local", "Ablation Study", Sec. 5.6): Eq. 3 and the warm-up branch applied to the
                                       model's norm; its single gamma lives in ema_norms[0] */
#define ADAGC_MODE_ZCLIP         3  /* ZClip, a baseline of the paper's comparison (Table 2: h = min{1, tau/||g||},
                                       tau = mu + xi(z) sigma, z = (||g|| - mu)/sigma on the model's norm; appendix
                                       "Clipping Hyper-Parameters": alpha 0.97, z_thres 2.0).  The paper leaves xi and
                                       the statistics' update undefined; this library takes xi(z) = z_thres^2 / z,
                                       active for z > z_thres, and feeds the clipped norm nhat to
                                       mu' = alpha mu + (1-alpha) nhat, var' = alpha var + (1-alpha)(nhat - mu')^2.
                                       alpha is ema_beta; mu lives in ema_norms[0], var in ema_norms[1] (so
                                       ema_norms needs at least 2 entries).  Steps 1..t_start only gather the
                                       statistics under GlobalGC (Eq. 2 with lambda_abs): step 1 sets mu to its
                                       clipped norm and var to 0 */

#define ADAGC_MODE_AGC           4  /* update clipping, Table 2's AGC row: the gradient is left alone and each tensor's
                                       update direction Delta (AdamW: mhat/(sqrt(vhat)+eps); Lion: sign(c)) is scaled by
                                       min{1, lambda_rel ||theta|| / ||Delta||} (l2 norms, theta before the step; the paper's
                                       setting: lambda_rel 1e-3).  One tensor of the list is one unit; weight decay is
                                       applied unscaled.  Needs adagc_config.update_clipping = 1; keeps no state;
                                       adagc_get_norms then reports ||Delta_i|| and the update's coefficient */
#define ADAGC_MODE_CLIPPY        5  /* update clipping, Table 2's Clippy row: the same with
                                       min{1, (lambda_rel ||theta||_inf + lambda_abs) / (lr ||Delta||_inf)}
                                       (the paper's setting: lambda_abs 0.5, lambda_rel 1e-2) */

typedef struct adagc_ctx adagc_ctx; /* opaque; created by adagc_create, freed by adagc_destroy */

/* One parameter tensor = one clipping unit (Sec. 4.2: "each parameter tensor";
 * a fused QKV weight is one tensor).  Only its element count matters. */
typedef struct {
    int64_t  numel;    /* > 0 */
    uint32_t flags;    /* must be 0 */
    uint32_t reserved; /* must be 0 */
} adagc_tensor_desc;

typedef struct {
    int32_t optimizer;            /* ADAGC_OPT_ADAMW or ADAGC_OPT_LION */
    int32_t grad_dtype;           /* ADAGC_GRAD_F32 or ADAGC_GRAD_BF16 (widened exactly in-kernel) */
    int32_t has_bf16_param_copy;  /* 1: every step also writes round-to-nearest-even bf16 copies of the
                                     updated params to the buffers given to adagc_set_param_copies */
    int32_t telemetry;            /* 1: every step also reduces, inside the update kernel, the per-tensor l2
                                     norms of the first moment, the second moment and the parameter update
                                     (the quantities the paper plots per tensor, Fig. 2); read them with
                                     adagc_get_state_norms.  Costs no extra HBM traffic. */
    /* Launch tuning of the streaming kernels; 0 = library default for each. */
    int32_t grid_blocks;          /* > 0: persistent grid of that many workgroups, each walking work items
                                     b, b+grid, ...; default: one work item per workgroup (a chunk in the
                                     norm kernel; a chunk or a part of one in the update kernel) */
    int32_t unroll;               /* 128-bit vectors per lane per array kept in flight by the update kernel:
                                     1, 2 or 4 (default 4) */
    int32_t nontemporal;          /* streaming (non-temporal) loads and stores: 1 = on (default), 2 = off */
    int32_t schedule;             /* visiting order of the chunks, see adagc_build_visiting_order: number of
                                     contiguous parts the list is cut into (default 2; 1 = list order) */
    int32_t update_split;         /* work items of the update kernel per chunk: 1 = whole chunks, or 2, 4, ...
                                     up to chunk_elems / (unroll*1024).  Default (0): 4096-element items
                                     (small items shorten the tail of the launch and give short lists more
                                     workgroups; whole chunks cost the fewest dispatches) */
    int32_t schedule_run;         /* visiting order: chunks an XCD takes in a row (default 8) */
    int32_t update_clipping;      /* 1: reserve the scratch the update-clipping modes need (ADAGC_MODE_AGC and
                                     ADAGC_MODE_CLIPPY: two extra partial results per work item of the update
                                     kernel); those modes return ADAGC_ERR_STATE without it */
} adagc_config;

/* Hyper-parameters of Alg. 1, passed by the caller on every step (the learning
 * rate schedule {eta_t} lives with the caller).  Defaults in the paper:
 * lambda_rel 1.04 and ema_beta 0.99 ("Critical Hyperparameter Selection", Sec. 5.2), t_start 100
 * (Sec. 4.2), lambda_abs 1.0 (appendix "Clipping Hyper-Parameters"). */
typedef struct {
    float   lr;            /* eta_t */
    float   beta1, beta2;  /* AdamW: moment decay rates.  Lion: interpolation / momentum rates */
    float   eps;           /* AdamW epsilon (added outside the square root); ignored by Lion */
    float   weight_decay;  /* lambda_w, decoupled, applied to every tensor */
    float   lambda_rel;    /* relative threshold of Eq. 3; +inf disables per-tensor clipping */
    float   ema_beta;      /* beta of the EMA in Eq. 3, in [0, 1) */
    float   lambda_abs;    /* GlobalGC threshold of the warm-up (Eq. 2); +inf disables it */
    int32_t t_start;       /* number of warm-up steps: steps 1..t_start take the warm-up branch.
                              0 = never: ema_norms must then be pre-filled by the caller.  Eq. 3 is applied as
                              printed, so a tensor whose gamma is 0 gets threshold 0, coefficient 0 (visible in
                              adagc_get_norms) and a gamma that stays 0: the warm-up branch is what initialises
                              gamma, and at least one warm-up step (t_start >= 1) is the intended use */
    int32_t clip_mode;     /* ADAGC_MODE_*; 0 = the paper's method */
    float   z_thres;       /* ADAGC_MODE_ZCLIP only: z-score threshold, > 0 (+inf: never clip); ignored otherwise */
} adagc_hyper;

/* Device-resident inputs of adagc_step_graph: the hyper-parameters and the step number are read by the
 * GPU when the step runs, not by the host when it is enqueued. */
typedef struct {
    adagc_hyper hp;
    int64_t     step;      /* 1-based t of Alg. 1 */
} adagc_step_params;

/* Elements per chunk of the segment table (a compile-time constant of the library). */
int64_t adagc_chunk_elems(void);

/*
 * Host-only: cut a tensor list into chunks.  Each tensor is cut at multiples of
 * chunk_elems counted from its own first element (the last chunk of a tensor is
 * ragged); chunks appear in list order.  Needs no GPU.
 *   descs        HOST  n_tensors descriptors
 *   chunk_begin  HOST  out, n_tensors+1 entries: index of each tensor's first chunk; last = total
 *   chunk_tensor HOST  out, capacity entries (may be NULL to only count): owning tensor of chunk c
 *   chunk_index  HOST  out, capacity entries (may be NULL): position of chunk c inside its tensor;
 *                      its first element is chunk_index*chunk_elems
 *   n_chunks     HOST  out: total number of chunks
 * Errors: INVALID_ARG (NULL descs/chunk_begin/n_chunks, n_tensors <= 0, chunk_elems <= 0,
 * numel <= 0, non-zero flags, capacity too small while arrays are given), TOO_LARGE.
 */
int adagc_build_segment_table(const adagc_tensor_desc* descs, int64_t n_tensors, int64_t chunk_elems,
                              int64_t* chunk_begin, uint32_t* chunk_tensor, uint32_t* chunk_index,
                              int64_t capacity, int64_t* n_chunks);

/*
 * Host-only: the order in which the streaming kernels visit the chunks.  Workgroups
 * are dealt to the GPU's 8 XCDs (each with its own L2) in turn, so position k of the
 * order is worked on by XCD k mod 8.  With parts in {1, 2, 4, 8} the list is cut into
 * that many contiguous parts, XCD x works in part x mod parts, and the 8/parts XCDs
 * that share a part take runs of `run` consecutive chunks in turn.  Any other parts
 * value deals position k to part k mod parts (run is ignored).  The order changes
 * which workgroup touches which chunk and when, never a result.
 *   order  HOST  out, n_chunks entries: a permutation of 0 .. n_chunks-1
 * Errors: INVALID_ARG (NULL, n_chunks/parts/run <= 0), TOO_LARGE.
 */
int adagc_build_visiting_order(int64_t n_chunks, int32_t parts, int32_t run, uint32_t* order);

/*
 * Create a context for a fixed tensor list on the current GPU: validates the
 * descriptors, builds the segment table, allocates and uploads it together with
 * the reduction scratch (one fp64 partial per chunk) and the per-tensor result
 * arrays.  All device memory the library ever needs is allocated here.
 *   out    HOST  receives the context (untouched on error)
 *   descs  HOST  n_tensors descriptors, copied
 *   cfg    HOST  copied
 */
int adagc_create(adagc_ctx** out, const adagc_tensor_desc* descs, int64_t n_tensors,
                 const adagc_config* cfg);

/* Free the context and its device memory.  The caller must make sure no step is still running. */
void adagc_destroy(adagc_ctx* ctx);

/*
 * Register the bf16 parameter copies (only with has_bf16_param_copy = 1).
 *   params_bf16  HOST array of n_tensors DEVICE pointers, tensor i holding numel_i bf16 values.
 * The array is copied; the buffers stay owned by the caller.
 */
int adagc_set_param_copies(adagc_ctx* ctx, void* const* params_bf16);

/*
 * One optimizer step (one pass of the loop body of Alg. 1) over the whole list,
 * enqueued on `stream`; allocates nothing and returns without waiting for the GPU.
 * (One bounded exception: the device pointers of the four arrays are mirrored on the
 * GPU and re-uploaded, through a ring of four pinned staging tables, only when they
 * differ from the previous call's.  A caller whose pointers change on every call and
 * who runs more than four such calls ahead of the GPU waits until the oldest of those
 * uploads has left its staging table.)
 *   params      HOST array of n_tensors DEVICE pointers, fp32, updated in place      (theta)
 *   grads       HOST array of n_tensors DEVICE pointers, fp32 or bf16 per cfg, read only   (g_t)
 *   exp_avg     HOST array of n_tensors DEVICE pointers, fp32, updated in place      (m)
 *   exp_avg_sq  HOST array of n_tensors DEVICE pointers, fp32, updated in place      (v); NULL for Lion
 *   ema_norms   DEVICE fp32[n_tensors], updated in place                              (gamma_i);
 *               ADAGC_MODE_GLOBAL_ADAGC uses element 0 only, ADAGC_MODE_GLOBALGC none,
 *               ADAGC_MODE_ZCLIP elements 0 and 1 (fp32[max(n_tensors, 2)])
 *   hp          HOST hyper-parameters of this step
 *   step        1-based t of Alg. 1: drives the bias correction and the warm-up test
 *   stream      hipStream_t (NULL = the default stream)
 * The host pointer arrays are read during the call and may be reused afterwards.
 * Pointers aligned to 16 bytes (8 for bf16 arrays) take the vectorised path; any
 * other alignment is accepted and handled element by element.
 * Non-finite gradients get no special treatment: a NaN norm compares false
 * against the threshold, so the tensor is not clipped and the NaN propagates as
 * it would in plain AdamW.
 * The update-clipping modes read g, theta, m, v once more instead of the norm pass (the direction's norms
 * must be complete before any element is updated): 16 + 30 bytes per parameter instead of 4 + 30.
 * Errors: INVALID_ARG, STATE (bf16 copies expected but not set; update clipping not reserved), HIP.
 */
int adagc_step(adagc_ctx* ctx, void* const* params, const void* const* grads,
               void* const* exp_avg, void* const* exp_avg_sq, float* ema_norms,
               const adagc_hyper* hp, int64_t step, void* stream);

/*
 * adagc_step for callers that record their work into a HIP graph: the same step, except that the
 * hyper-parameters and the step number come from DEVICE memory and are read when the kernels run.
 * A launch sequence recorded once (stream capture) can therefore be replayed for every later step;
 * between replays the caller updates *step_params (a copy or kernel of its own, ordered before the
 * replay).  Which branch of Alg. 1 applies (warm-up or not, clip_mode) is decided on the device, so
 * the recorded sequence is the same for all of them (six kernels where adagc_step launches three to five).
 *   step_params  DEVICE adagc_step_params, read by the GPU during the step
 *   other arguments as for adagc_step
 * The parameters cannot be validated on the host: a step whose parameters adagc_step would reject
 * leaves all state untouched, and the next adagc_get_norms / adagc_get_state_norms returns
 * INVALID_ARG (this includes the update-clipping modes, which this entry point does not offer).
 * The bias corrections use the device's pow(), which may differ from the host's in
 * the last bit of a double (invisible after rounding to fp32 in all but about one value in 10^8).
 * While `stream` is capturing, the call records kernels only: the tensor pointers must be the ones
 * of the previous call on this context (make one uncaptured call first; otherwise STATE), and
 * adagc_profile_begin must not be active.  Allocates nothing.
 * Errors: INVALID_ARG, STATE, HIP.
 */
int adagc_step_graph(adagc_ctx* ctx, void* const* params, const void* const* grads,
                     void* const* exp_avg, void* const* exp_avg_sq, float* ema_norms,
                     const adagc_step_params* step_params, void* stream);

/*
 * For callers that cannot allocate device memory: code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The same step as adagc_step, without a context:
 * this call allocates nothing (no hipMalloc / hipFree, no copy, no memset, no event), it only
 * launches kernels on `stream`.  The segment table, the per-chunk partial sums and the per-tensor
 * results live in a fixed array inside the library's device code, ADAGC_STATIC_MAX_* in size
 * (about 11 MB per GPU, held from the library's load until the process ends).
 *   descs, n_tensors, cfg   HOST  as for adagc_create; cfg->telemetry, cfg->update_clipping and the
 *                                 launch-tuning fields must be 0 (library defaults, chunks visited in
 *                                 list order; clip modes 0 to 3)
 *   params, grads, exp_avg, exp_avg_sq, ema_norms, hp, step, stream   as for adagc_step
 *   params_bf16   HOST array of n_tensors DEVICE pointers (cfg->has_bf16_param_copy = 1), else NULL
 *   out_norms     DEVICE fp32[n_tensors]  ||g_i|| before clipping        (may be NULL)
 *   out_coefs     DEVICE fp32[n_tensors]  h_i                            (may be NULL)
 *   out_clipped   DEVICE u8[n_tensors]    1 where the clip was active    (may be NULL)
 * The tensors belong to the current GPU.  Results are those of adagc_step bit for bit (the same
 * kernels; the visiting order never changes a result).
 * Limits: n_tensors <= ADAGC_STATIC_MAX_TENSORS and at most ADAGC_STATIC_MAX_CHUNKS chunks of
 * adagc_chunk_elems() elements (each tensor takes ceil(numel / chunk) of them); beyond that the call
 * returns ADAGC_ERR_TOO_LARGE and enqueues nothing.
 * Every call on a GPU uses that GPU's one array, whose contents are those of the last call: calls
 * that overlap on one GPU (two streams, two threads) race and must be ordered by the caller.  Nothing
 * in the array has to start at zero: each call overwrites every slot it reads.
 * Errors: INVALID_ARG, TOO_LARGE, HIP; arguments are validated before anything is enqueued.
 */
#define ADAGC_STATIC_MAX_TENSORS 32768
#define ADAGC_STATIC_MAX_CHUNKS  524288
int adagc_step_static(const adagc_tensor_desc* descs, int64_t n_tensors, const adagc_config* cfg,
                      void* const* params, const void* const* grads, void* const* exp_avg,
                      void* const* exp_avg_sq, void* const* params_bf16, float* ema_norms,
                      const adagc_hyper* hp, int64_t step, float* out_norms, float* out_coefs,
                      uint8_t* out_clipped, void* stream);

/*
 * Per-tensor results of the most recently enqueued step: copies them to the host
 * and waits for `stream`.  Any of the three output arrays may be NULL.
 *   host_norms    HOST fp32[n_tensors]   ||g_i|| before clipping
 *   host_coefs    HOST fp32[n_tensors]   h_i (the global h during warm-up)
 *   host_clipped  HOST u8[n_tensors]     1 where the clip was active
 *   n_tensors     must equal the context's tensor count
 */
int adagc_get_norms(adagc_ctx* ctx, float* host_norms, float* host_coefs, uint8_t* host_clipped,
                    int64_t n_tensors, void* stream);

/*
 * Telemetry of the most recently enqueued step (context created with telemetry = 1): per-tensor
 * l2 norms of the updated first moment m, of the updated second moment v (zeros for Lion) and of
 * the parameter update theta_t - theta_{t-1}, from the stored fp32 values.  Copies to the host
 * and waits for `stream`.  Any output may be NULL.  Errors: INVALID_ARG, STATE (telemetry off), HIP.
 */
int adagc_get_state_norms(adagc_ctx* ctx, float* host_m_norms, float* host_v_norms,
                          float* host_update_norms, int64_t n_tensors, void* stream);

/* Number of tensors / chunks of the context's segment table (negative error code for NULL). */
int64_t adagc_num_tensors(const adagc_ctx* ctx);
int64_t adagc_num_chunks(const adagc_ctx* ctx);

/*
 * Read the DEVICE-resident segment table back (synchronous), in the layout of
 * adagc_build_segment_table: chunk_begin HOST int64[n_tensors+1], chunk_tensor
 * and chunk_index HOST uint32[adagc_num_chunks].  Any may be NULL.
 */
int adagc_get_segment_table(adagc_ctx* ctx, int64_t* chunk_begin, uint32_t* chunk_tensor,
                            uint32_t* chunk_index);

/*
 * Per-kernel timing with HIP events on the step's own stream.
 * adagc_profile_begin reserves event slots for up to max_steps steps; every
 * following adagc_step records four events (before the norm kernel, after it,
 * after the per-tensor finalize, after the fused update).  adagc_profile_end
 * waits for the last recorded step, writes three durations per step in
 * milliseconds (norm, finalize, update) to ms (HOST float[3*max_steps]), the
 * number of recorded steps to n_steps, and releases the events.
 */
int adagc_profile_begin(adagc_ctx* ctx, int32_t max_steps);
int adagc_profile_end(adagc_ctx* ctx, float* ms, int32_t* n_steps);

/*
 * Muon with AdaGC's clipped gradient, for a context created with ADAGC_OPT_MUON (every tensor of the list a
 * matrix).  The paper pairs AdaGC with Muon ("Optimizer Compatibility: Muon and Lion", Sec. 5.4) and prints no
 * rule for it; this is the published one, with h_i g_i in the place of the gradient as Alg. 1 does for AdamW:
 *     M_i <- mu M_i + h_i g_i;   U = h_i g_i + mu M_i (nesterov) or M_i;
 *     X = U / (||U||_F + 1e-7), transposed if rows > cols;
 *     ns_steps times:  A = X X^T;  B = b A + c A A;  X <- a X + B X,   (a, b, c) = (3.4445, -4.7750, 2.0315),
 *         X, A, B stored as bf16, products on the matrix cores with fp32 accumulation;
 *     theta_i <- theta_i - lr (weight_decay theta_i + sqrt(max(1, rows/cols)) X).
 * h_i comes from the same norm pass and rule as in adagc_step (clip modes 0 to 3).
 */
typedef struct {
    int64_t rows, cols;        /* rows * cols = the tensor's numel; row-major */
} adagc_matrix_shape;

typedef struct {
    float   momentum;          /* mu in [0, 1); the published default is 0.95 */
    int32_t nesterov;          /* 1: U = h g + mu M (published default); 0: U = M */
    int32_t ns_steps;          /* Newton-Schulz steps, 0 to 16 (published default 5; 0 applies the normalised U itself) */
    int32_t reserved;          /* must be 0 */
} adagc_muon_hyper;

/*
 * Give the context the matrices' shapes and allocate the Newton-Schulz workspace.  Once per context.
 * Matrices whose extents, rounded up to multiples of 128, are equal are iterated together, up to 32 at a time
 * (fewer if 32 would need more than 24 GiB, or more than the device can give), by batched launches of the
 * matrix-core product: one launch over many matrices fills the GPU where one matrix has too few tiles.  The workspace (bf16) holds the largest such batch: per
 * matrix four copies of its padded min x max extent and two of min x min (adagc_muon_workspace_bytes tells the
 * total).  A matrix's result does not depend on which others share its batch.
 *   shapes  HOST  n_tensors entries, copied
 * Errors: INVALID_ARG (shape does not match numel), STATE (context not ADAGC_OPT_MUON, or attached already),
 * TOO_LARGE (a padded dimension beyond 2^31-1), OOM, HIP.
 */
int adagc_muon_attach(adagc_ctx* ctx, const adagc_matrix_shape* shapes);

/* Bytes of device workspace adagc_muon_attach allocated for this context (0 before it, or for a NULL context). */
int64_t adagc_muon_workspace_bytes(const adagc_ctx* ctx);

/*
 * One Muon step over the whole list, enqueued on `stream`; allocates nothing.
 *   params, grads, ema_norms, hp, step, stream   as for adagc_step (hp->beta1, beta2, eps are ignored;
 *                                                 hp->clip_mode 0 to 3)
 *   momentum   HOST array of n_tensors DEVICE pointers, fp32, updated in place      (M_i)
 *   mh         HOST Muon's own hyper-parameters
 * bf16 parameter copies are written if the context has them.
 * Errors: INVALID_ARG, STATE (not attached; copies expected but not set), HIP.
 */
int adagc_muon_step(adagc_ctx* ctx, void* const* params, const void* const* grads, void* const* momentum,
                    float* ema_norms, const adagc_hyper* hp, const adagc_muon_hyper* mh, int64_t step, void* stream);

/*
 * Building block of the Muon path, exported so that it can be checked on its own: the bf16 matrix-core
 * product of the Newton-Schulz iteration (the orthogonalisation step of Muon, the optimizer the paper pairs
 * AdaGC with in "Optimizer Compatibility: Muon and Lion", Sec. 5.4; the iteration itself is not printed there),
 *     C[i][j] = bf16( alpha * sum_k P[i][k] Q[j][k] + beta * D[i][j] ),   fp32 accumulation,
 * enqueued on `stream`.  All matrices DEVICE, bf16, row-major:
 *   P   M x K, leading dimension ldp        Q   N x K, ldq          (both operands K-contiguous)
 *   Dt  N x M, lddt: the TRANSPOSE of D, or NULL (then beta is ignored)
 *   C   M x N, ldc, or NULL                 Ct  N x M, ldct: the transpose of the result, or NULL (one of the two)
 *   symmetric = 1: P = Q, M = N and D symmetric, so the result is symmetric; it is written to Ct (C NULL or the same
 *                  array) and only the tiles on and below the diagonal are computed, each stored twice
 * M, N and K must be multiples of 128, every leading dimension of 8, every pointer 16-byte aligned.
 * Errors: INVALID_ARG, TOO_LARGE, HIP.
 */
int adagc_muon_gemm_nt(const void* P, int64_t ldp, const void* Q, int64_t ldq, int64_t M, int64_t N, int64_t K,
                       float alpha, float beta, const void* Dt, int64_t lddt, void* C, int64_t ldc, void* Ct,
                       int64_t ldct, int32_t symmetric, void* stream);

/*
 * The same product for `batch` (>= 1) sets of matrices of one shape in a single launch, as adagc_muon_step issues
 * it: matrix z of every array starts z * its stride (in elements, a multiple of 8, >= 0) after the pointer given.
 * strides  HOST array of 5: for P, Q, Dt, C, Ct in this order (entries of absent arrays are ignored; with
 *          symmetric = 1 the strides of P and Q must be equal).  The caller sees to it that the batch's outputs do
 *          not overlap.  Every matrix's result is the one adagc_muon_gemm_nt gives for it alone.
 * Errors: INVALID_ARG, TOO_LARGE, HIP.
 */
int adagc_muon_gemm_nt_batched(const void* P, int64_t ldp, const void* Q, int64_t ldq, int64_t M, int64_t N, int64_t K,
                               float alpha, float beta, const void* Dt, int64_t lddt, void* C, int64_t ldc, void* Ct,
                               int64_t ldct, int32_t symmetric, int64_t batch, const int64_t* strides, void* stream);

/* Static description of an error code. */
const char* adagc_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* ADAGC_H */
