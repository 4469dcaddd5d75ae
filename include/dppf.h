/*
 * dppf.h -- C ABI of the DPPF consensus-round library for AMD MI355X (gfx950).
 *
 * The library implements, for M workers whose fp32 parameter vectors x_1..x_M all live in
 * the memory of ONE GPU, the consensus round of Distributed Pull-Push Force and the local
 * optimizer step that runs between rounds:
 *
 *   x_A  = (1/M) sum_m x_m                              (Alg. 1, last line; Sec. 4)
 *   r_m  = || x_m - x_A ||_2   over the WHOLE model     (Alg. 1, push line; Eq. 5)
 *   x_m <- x_m + (x_A - x_m) * (alpha - lambda / r_m)   (Sec. 5, Eq. 5)
 *   v_m <- mu v_m + (g_m + wd x_m);  x_m <- x_m - eta v_m   (Alg. 1, SGD line, with the
 *                                     momentum 0.9 the experiments state in the appendix)
 *
 * Conventions common to every entry point
 *  - A model is a list of T tensors; worker m's copy of tensor t has numel[t] fp32 elements.
 *    The norm r_m runs over the concatenation of all T tensors.
 *  - "Pointer table" arguments are HOST arrays of DEVICE pointers.  Per-worker tables hold
 *    M*T entries, worker-major: table[m*T + t].  Per-model tables (x_A, x_C) hold T entries.
 *    The library copies a table to a plan-owned device buffer the first time it sees it and
 *    again only when its contents change; the host array may be freed after the call returns.
 *  - Every tensor pointer must be 4-byte aligned; nothing more is required (no 16-byte
 *    alignment, no padding, any numel >= 0).  Tensors must not overlap one another.
 *  - All tensors are owned by the caller.  x and v (and the Adam moments) are updated IN
 *    PLACE.  The library never allocates, frees or resizes caller memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    ENQUEUE work on it and return without waiting for the GPU.  A plan must not be used
 *    from two streams or two host threads at the same time (it owns scratch buffers and the
 *    counter its kernels take their work from); neither may a captured graph that uses a plan
 *    run at the same time as other work on that plan.
 *  - Calls may be captured into a HIP graph, provided one eager call with the same pointer
 *    tables was made before (a new table is uploaded with an event wait that capture forbids).
 *  - Small outputs r_out / c_out are DEVICE arrays of M floats, written by the enqueued work.
 *  - Return value: DPPF_OK (0) or a negative DPPF_E* code.  No exceptions, no aborts.
 *    Arguments are validated before anything is enqueued; on error nothing was launched.
 *  - A worker at distance zero (r_m == 0, e.g. identical replicas) is NOT an error: the
 *    direction of its push is undefined, its displacement is the zero vector, so its x_m is
 *    left bit-for-bit unchanged, r_m = 0 and c_m = alpha are reported.
 *  - pull (alpha) and push (lambda) are used as given: no clamping, no division by M.
 */
#ifndef DPPF_H_
#define DPPF_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DPPF_OK = 0,
  DPPF_EINVAL = -1,  /* bad argument: null required pointer, M < 1, T < 0, numel < 0,
                        misaligned tensor pointer, size mismatch with the plan            */
  DPPF_EHIP = -2,    /* a HIP runtime call failed; see dppf_last_hip_error()              */
  DPPF_ENOMEM = -3,  /* host or device allocation failed in dppf_plan_create              */
  DPPF_ELIMIT = -4   /* a size exceeds what the library supports (see DPPF_MAX_WORKERS)   */
};

#define DPPF_MAX_WORKERS 1024

/* Message for a return code (static storage, never NULL). */
const char* dppf_strerror(int code);
/* hipError_t (as int) of the most recent failed HIP call on this host thread, 0 if none. */
int dppf_last_hip_error(void);

/* ---------------------------------------------------------------------------------------
 * Plan: everything that depends only on the shape of the problem (M, the tensor sizes) --
 * the tile list that maps thread blocks to pieces of tensors, device copies of pointer
 * tables, the per-block partial sums of the norm reduction, the per-worker coefficients.
 * Creating a plan allocates device memory and synchronises; no later call does.
 * ------------------------------------------------------------------------------------- */
typedef struct dppf_plan dppf_plan;

/* numel: HOST array of T element counts.  Uses the HIP device that is current at the time of the
 * call; the same device must be current whenever the plan is used (a call made with another
 * device current returns DPPF_EINVAL and enqueues nothing).  */
int dppf_plan_create(dppf_plan** out, int M, int T, const int64_t* numel);
int dppf_plan_destroy(dppf_plan* plan);
/* d = sum of numel. */
int64_t dppf_plan_dim(const dppf_plan* plan);

/* HOST-ONLY, need no GPU: the work decomposition.  Every tensor is cut into tiles of at most
 * tile_elems consecutive elements; the list holds all full tiles first (in list order), then the
 * partial ones (tensor tails, small tensors).  The sweeps of the round use tiles of
 * dppf_sweep_tile_elems(M) elements (4096 up to 4 workers, 2048 up to 16, 1024 up to 39, 4096
 * beyond); the local steps always use DPPF_STEP_TILE_ELEMS.  dppf_layout_tiles writes d = sum
 * numel, the number of full tiles and the total; if the three tile arrays are non-NULL (capacity
 * `cap` entries, else DPPF_ELIMIT) also each tile's tensor index, first element inside that
 * tensor, and element count.  */
#define DPPF_STEP_TILE_ELEMS 4096
int dppf_sweep_tile_elems(int M);
int dppf_layout_tiles(int tile_elems, int T, const int64_t* numel, int64_t* d, int64_t* nfull, int64_t* ntiles,
                      int64_t cap, int32_t* tile_tensor, int64_t* tile_offset, int32_t* tile_count);

/* ---------------------------------------------------------------------------------------
 * Steps of the round (Alg. 1 consensus branch with x_C = x_A; Sec. 5 Eq. 5).
 * ------------------------------------------------------------------------------------- */

/* x_A[t][i] = (1/M) sum_m x[m][t][i].   x: M*T table (read).  xbar: T table (written). */
int dppf_replica_mean(dppf_plan* plan, const float* const* x, float* const* xbar, void* stream);

/* r_out[m] = || x_m - x_A ||_2.  xbar: T table holding x_A, or NULL to recompute it from x
 * on the fly (no extra memory traffic).  */
int dppf_dist_norms(dppf_plan* plan, const float* const* x, const float* const* xbar,
                    float* r_out, void* stream);

/* The whole round, Eq. 5, for all workers simultaneously from the same snapshot:
 *   c_m = pull - push / r_m  (pull if r_m == 0);  x_m <- x_m + (x_A - x_m) c_m.
 * r_out, c_out (device, M floats) and xbar_out (T table) are optional (NULL to skip) and
 * receive the distances, coefficients and average taken BEFORE the update.  */
int dppf_pull_push_round(dppf_plan* plan, float* const* x, float pull, float push,
                         float* r_out, float* c_out, float* const* xbar_out, void* stream);

/* ---------------------------------------------------------------------------------------
 * Local optimizer step between rounds (Alg. 1, SGD line; heavy-ball momentum, raw-gradient
 * buffer, coupled L2 weight decay):  g' = g + wd x;  v <- mu v + g';  x <- x - lr v.
 * x, v: M*T tables (read+written).  g: M*T table (read).
 * ------------------------------------------------------------------------------------- */
int dppf_local_sgd_step(dppf_plan* plan, float* const* x, float* const* v,
                        const float* const* g, float lr, float momentum, float weight_decay,
                        void* stream);

/* Fused: dppf_local_sgd_step followed by dppf_pull_push_round, with the step folded into the
 * round's first sweep so x is read one time less.  Same arithmetic per element; the squared
 * distances may be summed in a different order than in the two separate calls (the grids can
 * differ), so r_m agrees to rounding and everything else follows from it.  */
int dppf_round(dppf_plan* plan, float* const* x, float* const* v, const float* const* g,
               float lr, float momentum, float weight_decay, float pull, float push,
               float* r_out, float* c_out, float* const* xbar_out, void* stream);

/* ---------------------------------------------------------------------------------------
 * Variants of the round.
 * ------------------------------------------------------------------------------------- */

/* The round with the EXACT gradient of the relaxed Inverse-Mean-Valley regulariser, both terms
 * of Eq. 4 (a) kept (appendix "Ablation Study on the Second Term"):
 *   d_m = x_m - x_A;  x_m <- x_m - pull d_m + (push_r / M^2) (M d_m/||d_m|| - sum_j d_j/||d_j||).
 * push_r is the regulariser's own coefficient lambda_r (Eq. 5's lambda corresponds to push_r / M).
 * Workers at zero distance contribute a zero unit vector.  The average of the workers is
 * preserved.  r_out[m] = ||d_m||, c_out[m] = pull - (push_r/M)/r_m, both optional.  Up to 39
 * workers the same two sweeps and the same memory traffic as dppf_pull_push_round; for more workers
 * the average and the sum of unit vectors are staged in two plan-owned d-vectors.  */
int dppf_pull_push_round_exact(dppf_plan* plan, float* const* x, float pull, float push_r,
                               float* r_out, float* c_out, void* stream);

/* Alg. 1 taken literally, for ANY consensus variable x_C supplied by the caller (T table, read):
 *   x_m <- (1 - pull) x_m + pull x_C;  then  x_m <- x_m + push (x_m - ref) / ||x_m - ref||
 * with the ALREADY PULLED x_m, where ref is the workers' average before the round
 * (DPPF_PUSH_FROM_AVERAGE, Alg. 1) or x_C itself (DPPF_PUSH_FROM_CONSENSUS, the variant the
 * appendix remark on leader-based consensus describes).  A worker whose pulled gap is zero gets
 * no push.  r_post_out[m] (optional) = norm of the pulled gap.  With x_C = x_A and pull < 1 the
 * result equals dppf_pull_push_round.  */
enum { DPPF_PUSH_FROM_AVERAGE = 0, DPPF_PUSH_FROM_CONSENSUS = 1 };
int dppf_pull_then_push(dppf_plan* plan, float* const* x, const float* const* x_c, float pull,
                        float push, int push_from, float* r_post_out, void* stream);

/* AdamW local step (the optimizer of the ViT experiments, appendix; formula: decoupled weight
 * decay Adam):  x <- x (1 - lr wd);  m1 <- b1 m1 + (1-b1) g;  m2 <- b2 m2 + (1-b2) g^2;
 *   x <- x - lr (m1 / (1-b1^step)) / (sqrt(m2 / (1-b2^step)) + eps),   step = 1, 2, ...
 * x, m1, m2: M*T tables (read+written); g: M*T table (read).  */
int dppf_local_adamw_step(dppf_plan* plan, float* const* x, float* const* m1, float* const* m2,
                          const float* const* g, float lr, float beta1, float beta2, float eps,
                          float weight_decay, int64_t step, void* stream);

/* Fused: dppf_local_adamw_step followed by dppf_pull_push_round, with the step folded into the
 * round's first sweep (x is read one time less: 36 instead of 40 bytes per replica-parameter;
 * same remark on the summation order as for dppf_round).  r_out, c_out optional.  */
int dppf_round_adamw(dppf_plan* plan, float* const* x, float* const* m1, float* const* m2,
                     const float* const* g, float lr, float beta1, float beta2, float eps,
                     float weight_decay, int64_t step, float pull, float push, float* r_out,
                     float* c_out, void* stream);

/* ||x_A||_2, the Euclidean norm of the workers' average (appendix "DPPF's Hyperparameter
 * Sensitivity ..." tracks it next to the valley width): every round enqueued on a plan
 * (dppf_pull_push_round, dppf_round, dppf_pull_push_round_exact, dppf_round_adamw) leaves the norm
 * of the average it formed -- taken before the update, like r_out -- in the plan; this call
 * enqueues a copy of it to out (DEVICE, 1 float).  It costs the round no extra memory traffic.  */
int dppf_plan_average_norm(dppf_plan* plan, float* out, void* stream);

/* What the paper logs every round (appendix "Pull-Push Mechanism"), from the distances r (device,
 * M floats, e.g. r_out of a round):  out[0] = relaxed MV = (1/M) sum_m r_m (the valley width);
 * out[1..M] = pull strength pull*r_m;  out[M+1..2M] = push strength push.  With avg_norm (device,
 * 1 float, e.g. from dppf_plan_average_norm; NULL to skip) also out[2M+1] = ||x_A|| and
 * out[2M+2] = valley width / ||x_A|| (appendix, hyper-parameter sensitivity).
 * out: device, 2M+3 floats.  */
int dppf_round_statistics(const float* r, int M, float pull, float push, const float* avg_norm, float* out,
                          void* stream);

/* Push-strength schedules (appendix "How to Schedule The Pushing Force?"), a HOST function:
 * fixed: push;  decreasing: (push/2)(1 + cos(pi t/t_total));  increasing: (push/2)(1 - cos(pi t/t_total)). */
enum { DPPF_SCHEDULE_FIXED = 0, DPPF_SCHEDULE_DECREASING = 1, DPPF_SCHEDULE_INCREASING = 2 };
float dppf_push_schedule(int kind, float push, int64_t t, int64_t t_total);

/* ---------------------------------------------------------------------------------------
 * Flat convenience forms for a plan made with T == 1: worker m's vector starts at
 * x + m*ld (ld >= d elements).  Same semantics as the table forms above.
 * ------------------------------------------------------------------------------------- */
int dppf_pull_push_round_flat(dppf_plan* plan, float* x, int64_t ld, float pull, float push,
                              float* r_out, float* c_out, float* xbar_out, void* stream);
int dppf_local_sgd_step_flat(dppf_plan* plan, float* x, float* v, const float* g, int64_t ld,
                             float lr, float momentum, float weight_decay, void* stream);
int dppf_round_flat(dppf_plan* plan, float* x, float* v, const float* g, int64_t ld,
                    float lr, float momentum, float weight_decay, float pull, float push,
                    float* r_out, float* c_out, float* xbar_out, void* stream);

/* ---------------------------------------------------------------------------------------
 * For callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: dppf_pull_push_round_flat without a plan.
 * Same arithmetic and same kernels as dppf_pull_push_round_flat (x: DEVICE, worker m's vector
 * of d floats starts at x + m*ld, ld >= d, updated in place; r_out, c_out: DEVICE, M floats,
 * optional), but every buffer a plan would own -- tile list, pointer table, partial sums,
 * work counter -- lives in a device array of DPPF_STATIC_SCRATCH_BYTES bytes that is part of
 * the library image (each GPU the library is used on holds its own copy until the process
 * ends).  The call allocates nothing on the device and nothing on the host, copies nothing
 * from host memory and issues no memset: it enqueues kernels only.
 * Limits: M <= DPPF_STATIC_MAX_WORKERS and d <= DPPF_STATIC_MAX_DIM, else DPPF_ELIMIT and
 * nothing is enqueued.  All calls on one GPU share that GPU's array, which keeps the last
 * call's contents (each call rewrites what it reads): two such calls that could overlap on one
 * GPU (different streams, or two threads) race and must be serialised by the caller.
 * ------------------------------------------------------------------------------------- */
#define DPPF_STATIC_MAX_WORKERS 16
#define DPPF_STATIC_MAX_DIM 134217728            /* 2^27 elements per worker */
#define DPPF_STATIC_SCRATCH_BYTES 1328384
int dppf_pull_push_round_flat_static(float* x, int M, int64_t d, int64_t ld, float pull, float push,
                                     float* r_out, float* c_out, void* stream);

/* ---------------------------------------------------------------------------------------
 * Per-kernel timing with HIP events on the caller's stream (for benchmarks).  While
 * enabled, every kernel the plan launches is bracketed by two events.  dppf_plan_timing_read
 * waits for the recorded work, then returns up to `cap` records of the launches made since
 * the last read: kernel_id[i] (DPPF_K_*) and ms[i].  Returns the number of records, or a
 * negative error code.  Disabled by default; when disabled nothing is recorded.
 * ------------------------------------------------------------------------------------- */
enum {
  DPPF_K_REDUCE = 0,       /* sweep 1 of the round: average + squared distances          */
  DPPF_K_STEP_REDUCE = 1,  /* sweep 1 of the fused round: local step (v stored, x not)
                              + average + distances                                      */
  DPPF_K_FINALIZE = 2,     /* partial sums -> r_m, c_m                                   */
  DPPF_K_UPDATE = 3,       /* sweep 2 of the round: Eq. 5                                */
  DPPF_K_LOCAL_STEP = 4,   /* stand-alone local step                                     */
  DPPF_K_MEAN = 5,         /* stand-alone average                                        */
  DPPF_K_STEP_UPDATE = 6,  /* sweep 2 of the fused round: x - lr v rebuilt, then Eq. 5   */
  DPPF_K_UPDATE_EXACT = 7, /* sweep 2 with the two-term gradient                         */
  DPPF_K_SEQ_REDUCE = 8,   /* dppf_pull_then_push, sweep 1                               */
  DPPF_K_SEQ_UPDATE = 9,   /* dppf_pull_then_push, sweep 2                               */
  DPPF_K_ADAMW_STEP = 10,  /* AdamW local step                                           */
  DPPF_K_ADAMW_REDUCE = 11 /* sweep 1 of the fused AdamW round                           */
};
int dppf_plan_timing_enable(dppf_plan* plan, int enable);
int dppf_plan_timing_read(dppf_plan* plan, int* kernel_id, float* ms, int cap);

#ifdef __cplusplus
}
#endif
#endif /* DPPF_H_ */
