/*
 * fda.h -- C ABI of the FDA (Federated Dynamic Averaging, arxiv 2405.20988) monitor for
 * K simulated workers held as one [K, d] parameter slab in the memory of ONE AMD
 * MI355X (gfx950).
 *
 * What the library computes, per training step (Algorithm 1, lines 6-9):
 *   line 6  fda_local_state        the K local states S_k = (||u_k||^2, <xi,u_k>, sk(u_k))
 *                                  of the drifts u_k = w_k - w_t0 (Section 3; Thm 1; Thm 2)
 *   line 7-8 fda_estimate_variance the averaged state, the two variance over-estimates
 *                                  H(S) and their comparison with the threshold Theta
 *   line 9  fda_sync               w_k <- mean_k w_k for every worker, in place
 *           fda_update_xi          the LinearFDA direction from the last two synchronized
 *                                  models (Section 3.2, last display)
 *
 * Conventions
 *   - C99, no C++ types, nothing is thrown, nothing aborts.  Every call returns FDA_OK (0)
 *     or a negative FDA_E* code; fda_strerror() names it and fda_last_error() gives the
 *     detail of the most recent failure on the calling thread.
 *   - "DEVICE" pointers are addresses in the current HIP device's memory; "HOST" pointers
 *     are ordinary process memory.  The library allocates no device memory and frees
 *     none: slab, vectors, states, result structs and the workspace belong to the caller
 *     (for example torch tensors) and must stay alive until the work enqueued on `stream`
 *     has completed.  The library keeps no caller pointer after a call returns, except
 *     the workspace given to fda_create, which it uses until fda_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All calls
 *     only enqueue work, except fda_estimate_variance with a non-NULL out_host, which
 *     also waits for the stream.
 *   - One fda_ctx serves one stream at a time (its workspace is scratch for the kernels).
 *   - Without a usable HIP device every call that needs one fails with FDA_EHIP; there is
 *     no CPU fallback.
 */
#ifndef FDA_H_
#define FDA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* error codes */
#define FDA_OK       0
#define FDA_EINVAL  (-1)   /* NULL pointer, non-positive size, bad enum, misaligned pointer     */
#define FDA_ERANGE  (-2)   /* d not below the hash prime, sketch too large for one CU's LDS ... */
#define FDA_ENOMEM  (-3)   /* workspace smaller than fda_workspace_bytes() asks for             */
#define FDA_EHIP    (-4)   /* a HIP runtime call failed (no device, bad launch, ...)            */

/* storage type of the slab elements; w_t0, w_prev, xi and the states are always fp32 */
#define FDA_F32   0
#define FDA_BF16  1        /* bfloat16: drift and every accumulation are formed in fp32  */

/* which state components / estimates to produce (bit mask) */
#define FDA_VARIANT_LINEAR  1   /* LinearFDA, Thm 2 */
#define FDA_VARIANT_SKETCH  2   /* SketchFDA, Thm 1 */

#define FDA_MAX_SKETCH_ROWS 16
#define FDA_HASH_PRIME      2147483647u   /* 2^31 - 1 */

typedef struct fda_ctx fda_ctx;   /* opaque */

/*
 * Problem description (Section 3, "Problem formulation" and "Notation": K workers, each a
 * model w_k in R^d; Section 3.1: an l x m AMS sketch with error parameter eps).
 *
 * hash_coef: HOST pointer to l*2*4 uint32 values, index [row][which][e], every value
 * below 2^31 - 1.  Row i of the sketch uses two cubic polynomials over the prime
 * p = 2^31 - 1,  g(j) = c3 j^3 + c2 j^2 + c1 j + c0 mod p  with c_e = hash_coef[i][which][e]:
 * which = 0 places coordinate j in bucket floor(g(j) * m / 2^31); which = 1 gives its sign,
 * +1 if g(j) is even and -1 otherwise.  The values are copied by fda_create.  May be NULL
 * when FDA_VARIANT_SKETCH is not requested.
 */
/* fda_desc.flags: keep every sketch row in its own slot of the tabulated hash (no placement against
 * LDS collisions, see fda_plan_info.placed_row_group): same results bit for bit, a slower state pass --
 * for comparisons */
#define FDA_DESC_PLAIN_TABLE 1

typedef struct fda_desc {
  int32_t K;            /* number of workers (rows of the slab), >= 1                      */
  int32_t dtype;        /* FDA_F32 or FDA_BF16                                              */
  int64_t d;            /* model dimension, 1 <= d < 2^31 - 1 - 64                          */
  int64_t row_stride;   /* elements between consecutive rows of the slab, >= d              */
  int32_t variants;     /* FDA_VARIANT_* bit mask, non-zero                                 */
  int32_t l;            /* sketch rows,   1..FDA_MAX_SKETCH_ROWS (ignored without SKETCH)   */
  int32_t m;            /* sketch columns, >= 1                  (ignored without SKETCH)   */
  int32_t flags;        /* FDA_DESC_* bit mask, normally 0                                  */
  double  eps;          /* the epsilon of Thm 1: H = mean||u||^2 - M2 / (1 + eps)           */
  const uint32_t* hash_coef;
} fda_desc;

/* Result of fda_estimate_variance (64 bytes).  Entries of a variant that was not requested
 * are zero. */
typedef struct fda_estimate {
  double  mean_sqnorm;      /* (1/K) sum_k ||u_k||^2                                        */
  double  mean_proj;        /* (1/K) sum_k <xi,u_k>                                         */
  double  m2;               /* M2( (1/K) sum_k sk(u_k) ): median of the squared row norms   */
  double  h_linear;         /* Thm 2: mean_sqnorm - mean_proj^2                             */
  double  h_sketch;         /* Thm 1: mean_sqnorm - m2 / (1 + eps)                          */
  int32_t sync_linear;      /* 1 iff h_linear > theta (strict), or h_linear is not finite   */
  int32_t sync_sketch;      /* 1 iff h_sketch > theta (strict), or h_sketch is not finite   */
  int32_t near_tie_linear;  /* 1 iff |h_linear - theta| <= tie_tol * max(mean_sqnorm,|theta|) */
  int32_t near_tie_sketch;  /* same for h_sketch                                            */
  int32_t nonfinite;        /* 1 iff a requested estimate is NaN or infinite                */
  int32_t state_path;       /* which kind of sketch cell the context's last state pass ended up
                               using, read on the device when the estimate ran (no stream wait):
                               after fda_local_state 0 / 1 / 2 as fda_last_state_path reports,
                               after fda_mean_state 0 / 1 as fda_last_mean_state_path reports;
                               -1 without a sketch and from fda_estimate_variance_static          */
} fda_estimate;

/* How the state pass is laid out on the chip; filled by fda_plan (for inspection and for
 * sizing the workspace without a device). */
typedef struct fda_plan_info {
  int32_t worker_groups;    /* the K workers are split into this many groups of workgroups  */
  int32_t workers_per_group;/* largest group                                                */
  int32_t row_groups;       /* the l sketch rows are split into this many groups            */
  int32_t rows_per_group;   /* largest group                                                */
  int32_t partitions;       /* coordinate partitions (workgroups per worker group)          */
  int32_t threads;          /* threads per workgroup                                        */
  int64_t chunk;            /* coordinates per partition                                    */
  int64_t lds_bytes;        /* LDS per workgroup                                            */
  int64_t workspace_bytes;  /* device scratch the context needs                             */
  int64_t state_floats;     /* floats per worker state: 2 + l*m with SKETCH, else 2         */
  /* the mean-state pass (fda_mean_state): every workgroup reads all K workers */
  int32_t mean_row_groups;       /* sketch-row groups (1 unless l*m 8-byte cells exceed LDS)  */
  int32_t mean_rows_per_group;   /* largest group                                            */
  int32_t mean_partitions;       /* coordinate partitions                                    */
  int32_t mean_workgroups_per_cu;/* resident workgroups per CU the launch is sized for       */
  int64_t mean_chunk;            /* coordinates per partition                                */
  int64_t mean_lds_bytes;        /* LDS per workgroup                                        */
  int32_t sign_split_rows;  /* 1: the state pass keeps terms of sign -1 in LDS rows of their own */
  int32_t worker_slots;     /* worker slots of the state kernel that runs (>= workers_per_group)  */
  int32_t placed_row_group; /* rows per placement group of the tabulated hash (0: every row keeps its slot): the
                               slot of a record that holds a row is chosen per coordinate against LDS collisions */
  int32_t reserved;
} fda_plan_info;

const char* fda_strerror(int code);
/* Detail text of the last failing call on this thread (valid until the next failure). */
const char* fda_last_error(void);

/* Pure host computation: validate `desc` and lay out the state pass for a device with
 * `compute_units` CUs and `lds_bytes_per_cu` bytes of LDS per CU.  Touches no device. */
int fda_plan(const fda_desc* desc, int32_t compute_units, int64_t lds_bytes_per_cu,
             fda_plan_info* out);

/* Bytes of DEVICE scratch fda_create needs for `desc` on the current HIP device. */
int fda_workspace_bytes(const fda_desc* desc, size_t* bytes);

/* Create a context on the current HIP device.  `workspace` is a DEVICE pointer, 256-byte
 * aligned, of at least fda_workspace_bytes() bytes, owned by the caller and left with the
 * context until fda_destroy.  On failure *ctx is set to NULL.
 * All calls of one context use that workspace for their partial results: enqueue them on one
 * stream (or order them yourself); calls of one context that overlap on the device race.  A
 * context is used by one host thread at a time, with the device it was created on current
 * (anything else is FDA_EINVAL). */
int fda_create(fda_ctx** ctx, const fda_desc* desc, void* workspace, size_t workspace_bytes);
int fda_destroy(fda_ctx* ctx);

/* Floats per worker state S: state[k] = { ||u_k||^2, <xi,u_k>, sk(u_k) row-major l x m }.
 * (Thm 1: S_k in R x R^{l x m}; Thm 2: S_k in R x R; both share the first component.) */
int fda_state_floats(const fda_ctx* ctx, int64_t* S);
int fda_get_plan(const fda_ctx* ctx, fda_plan_info* out);

/*
 * Algorithm 1, line 6, for all K workers at once.
 *   w      DEVICE [K][row_stride] slab of dtype elements (row k = model of worker k)
 *   w_t0   DEVICE [d] fp32: the model after the most recent synchronization
 *   xi     DEVICE [d] fp32: the LinearFDA unit vector (may be NULL without LINEAR)
 *   state  DEVICE [K][S] fp32, written:  state[k][0] = ||w_k - w_t0||^2,
 *          state[k][1] = <xi, w_k - w_t0> (0 without LINEAR),
 *          state[k][2 + i*m + b] = sum over coordinates j in bucket b of row i of
 *          sign_i(j) (w_kj - w_t0_j)   (absent without SKETCH)
 * Pointers need the alignment of their element type only (2 bytes for a bf16 slab, 4 for everything
 * fp32; anything less is FDA_EINVAL): whole-vector loads are used for any d and any row_stride.
 * Sketch cells are accumulated as integers (a drift u enters as round(u * 2^e), 2^e chosen
 * per call so that the rounding is at most 2^-18 of the mean |u|), and everything across
 * workgroups is merged in a fixed order: with the integer cells (fda_last_state_path 0 or 1) the
 * state is bit-identical from run to run; the fp64 cells of the last fallback (path 2, and path 1
 * of fda_mean_state) add in the order the lanes arrive and are not.
 * The pass works on drifts scaled by that 2^e, so a single drift 2^45 times the mean magnitude or
 * more makes ||u_k||^2 overflow to infinity (reported as a non-finite estimate) where the plain
 * fp32 square would overflow only at 2^64.
 * The first call of a context also tabulates the hash into the workspace (one record per coordinate:
 * 11 bits per sketch row, 16 for m > 1024, 13 where the rows are placed -- fda_plan_info.placed_row_group --
 * rounded up to whole 16-bit words; 12 bytes for l = 7, m = 1000).  fda_mean_state tabulates a plain
 * table of its own on its first call when this pass uses placed rows.
 */
int fda_local_state(fda_ctx* ctx, const void* w, const float* w_t0, const float* xi,
                    float* state, void* stream);

/*
 * Algorithm 1, lines 7-8: average the K states, evaluate H of Thm 1 and/or Thm 2 in
 * fp64, compare with theta (strict '>').  tie_tol sets the near-tie flags (pass 1e-5 for
 * the tolerance the fp32 states are good for, 0 to flag exact ties only).
 *   state     DEVICE [K][S] as written by fda_local_state
 *   out_dev   DEVICE fda_estimate, written (required)
 *   out_host  HOST fda_estimate or NULL; if given the call copies the result and waits
 *             for `stream`
 */
int fda_estimate_variance(fda_ctx* ctx, const float* state, double theta, double tie_tol,
                          fda_estimate* out_dev, fda_estimate* out_host, void* stream);

/*
 * Algorithm 1, line 7 without line 6: the AVERAGE state of the K workers, computed directly.
 * With all workers in one address space the linearity of the sketch (Section 3.1,
 * sk(a u + b v) = a sk(u) + b sk(v)) and of the inner product give
 *   mean_state[0] = (1/K) sum_k ||u_k||^2,
 *   mean_state[1] = <xi, u_bar> = (1/K) sum_k <xi,u_k>,
 *   mean_state[2 + i*m + b] = sk(u_bar)[i][b] = (1/K) sum_k sk(u_k)[i][b],   u_bar = (1/K) sum_k u_k,
 * i.e. exactly the average of the K states fda_local_state writes, at l instead of l*K sketch
 * additions per coordinate.  Use it when the per-worker states themselves are not needed (they
 * are what a worker of a distributed run would send; one device holding all workers only needs
 * their mean).
 *   w, w_t0, xi   as in fda_local_state
 *   mean_state    DEVICE [S] fp32, written
 *   w_bar         DEVICE [d] fp32 or NULL.  If given it receives the average model
 *                 w_t0 + u_bar (what Algorithm 1 line 9 would install: the same pass has every
 *                 worker's element in registers anyway; 4 more bytes written per coordinate),
 *                 and the context keeps ||w_bar - w_t0||^2 for fda_sync_from_mean.
 * A drift enters the sketch as the integer round(u * 2^e) (2^e as in fda_local_state), the K
 * integers of a coordinate are summed and added to 64-bit cells: exact, hence bit-identical
 * from run to run; drifts beyond 2^11 times the sampled mean |u| send the call down an fp64 path.
 * Returns FDA_ERANGE if K times the coordinates per workgroup reaches 2^33.
 */
int fda_mean_state(fda_ctx* ctx, const void* w, const float* w_t0, const float* xi,
                   float* mean_state, float* w_bar, void* stream);

/*
 * Algorithm 1, line 8 on an average state: as fda_estimate_variance, but `mean_state` is the
 * DEVICE [S] vector fda_mean_state wrote (no averaging left to do).
 */
int fda_estimate_variance_mean(fda_ctx* ctx, const float* mean_state, double theta, double tie_tol,
                               fda_estimate* out_dev, fda_estimate* out_host, void* stream);

/*
 * fda_estimate_variance for callers that cannot allocate and hold no context: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernel and same result as
 * fda_estimate_variance (out_dev is written bit for bit the same, except state_path = -1: there is
 * no context whose last state pass could be reported), but the per-workgroup partial sums
 * and the finished-workgroup counter live in a static device array of the library (17 KiB per GPU,
 * held until the process ends) instead of a context's workspace.  Calls no hipMalloc / hipFree and no
 * allocating library routine, creates no events, never waits; enqueues a one-workgroup fill kernel
 * (the counter) and the estimate kernel on `stream`.
 *   state     DEVICE [K][S] fp32, S = 2 + l*m with FDA_VARIANT_SKETCH, else 2 (l, m then ignored)
 *   K >= 1;  l in 1..FDA_MAX_SKETCH_ROWS and m in 1..FDA_STATIC_MAX_M: larger is FDA_ERANGE
 *   variants, eps, theta, tie_tol, out_dev as in fda_create / fda_estimate_variance
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race; order them.  (K = 1 with a mean state gives fda_estimate_variance_mean.)
 */
#define FDA_STATIC_MAX_M 32767
int fda_estimate_variance_static(const float* state, int32_t K, int32_t l, int32_t m, int32_t variants,
                                 double eps, double theta, double tie_tol, fda_estimate* out_dev,
                                 void* stream);

/*
 * Algorithm 1, line 9 ("In-place"): every row of the slab becomes the average model.
 *   w        DEVICE slab, rewritten: row k <- (1/K) sum_k' row k'  (fp32 sum in worker
 *            order, divided by K; bf16 slabs store its round-to-nearest-even)
 *   w_t0     DEVICE [d] fp32, rewritten with the fp32 average
 *   w_prev   DEVICE [d] fp32 or NULL: receives the old w_t0 (the model after the second
 *            most recent synchronization, Table "Notation")
 *   pred_dev DEVICE int32 or NULL: if given and *pred_dev == 0 when the kernel runs,
 *            nothing is written (lets a step be enqueued without reading the decision
 *            back; point it at fda_estimate.sync_linear or .sync_sketch)
 */
int fda_sync(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, const int32_t* pred_dev,
             void* stream);

/*
 * Algorithm 1, line 9 followed by Section 3.2: fda_sync, then xi <- (w_t0 - w_prev) / ||w_t0 - w_prev||_2
 * for the new w_t0 and the old one (now in w_prev) -- what fda_sync followed by fda_update_xi computes,
 * except that the synchronization pass, which holds both models of every coordinate anyway, leaves
 * the squared norm of their difference, so that the refresh of xi is one pass over the two vectors
 * instead of two.  (The norm is the same sum of the same fp32 terms, added up in another fixed order:
 * xi agrees with fda_update_xi's to the last bit or two.)
 *   w, w_t0, pred_dev as in fda_sync;  w_prev and xi: DEVICE [d] fp32, both required
 */
int fda_sync_xi(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi, const int32_t* pred_dev,
                void* stream);

/*
 * Algorithm 1, line 9 and Section 3.2 in one write-only pass, for a caller whose last
 * fda_mean_state of this context produced `w_bar` from the slab as it still is:
 *   w        DEVICE slab, rewritten: every row <- w_bar (bf16 slabs: round-to-nearest-even)
 *   w_prev   DEVICE [d] fp32 or NULL: receives the old w_t0
 *   w_t0     DEVICE [d] fp32: <- w_bar
 *   xi       DEVICE [d] fp32 or NULL: <- (w_bar - old w_t0) / ||w_bar - old w_t0||_2, zero vector
 *            when the norm is zero or not finite (the norm is the one fda_mean_state left)
 *   w_bar    DEVICE [d] fp32 as written by fda_mean_state
 *   pred_dev as in fda_sync
 * Differs from fda_sync + fda_update_xi only in how the average was rounded (w_t0 + mean drift
 * instead of the sum of the rows divided by K; both within 1e-5 of the largest |w_kj|) and in
 * never reading the slab.
 */
int fda_sync_from_mean(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi,
                       const float* w_bar, const int32_t* pred_dev, void* stream);

/*
 * Section 3.2: xi <- (w_t0 - w_prev) / ||w_t0 - w_prev||_2 (all DEVICE [d] fp32); the zero
 * vector when the norm is zero or not finite.  pred_dev as in fda_sync.
 */
int fda_update_xi(fda_ctx* ctx, const float* w_t0, const float* w_prev, float* xi,
                  const int32_t* pred_dev, void* stream);

/*
 * Algorithm 1, lines 6-9 as one enqueue with no host round trip: the state, the estimate, and --
 * predicated on the device-side decision of the variant `decide_by` -- the synchronization and
 * the refresh of xi.  Exactly the calls above, in order:
 *   flags == 0:                    fda_local_state(state[K][S]), fda_estimate_variance,
 *                                  fda_sync_xi (fda_sync when xi == NULL)
 *   flags & FDA_STEP_MEAN_STATE:   fda_mean_state(state[S]), fda_estimate_variance_mean, then
 *                                  fda_sync_xi, or, with w_bar != NULL (which
 *                                  fda_mean_state then fills), fda_sync_from_mean
 *   decide_by   FDA_VARIANT_LINEAR or FDA_VARIANT_SKETCH (must be one of the context's variants)
 *   xi          read by the state pass (if LINEAR) and rewritten when the step synchronizes; with
 *               xi == NULL (allowed without LINEAR) no xi is maintained
 *   w_prev      DEVICE [d] fp32, required when xi is given
 *   w_bar       DEVICE [d] fp32 or NULL (only used with FDA_STEP_MEAN_STATE)
 *   out_dev / out_host  as in fda_estimate_variance (out_host != NULL makes the call wait)
 */
#define FDA_STEP_MEAN_STATE 1
int fda_step(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi, float* state, float* w_bar,
             double theta, double tie_tol, int32_t decide_by, int32_t flags, fda_estimate* out_dev,
             fda_estimate* out_host, void* stream);

/*
 * Diagnostic: which kind of LDS sketch cell the last fda_local_state of this context ended
 * up using -- 0: 32-bit integers (the normal case), 1: 64-bit integers (a drift was too large
 * for, or a sum did not fit, the 32-bit cells), 2: fp64 (the drifts' dynamic range is beyond
 * the 64-bit cells), -1: the context has no sketch.  Waits for `stream`.  The result of
 * fda_local_state is the same within the stated tolerance whichever path ran; only the time
 * differs.
 */
int fda_last_state_path(fda_ctx* ctx, int32_t* path, void* stream);
/* The same for the last fda_mean_state: 0: integer sums in 64-bit cells, 1: fp64, -1: no sketch. */
int fda_last_mean_state_path(fda_ctx* ctx, int32_t* path, void* stream);

/*
 * Measurement aid (no part of the method): when enabled, fda_local_state and fda_mean_state
 * bracket their streaming kernel -- the pass over the slab, Algorithm 1 line 6 -- with HIP
 * events on the caller's stream.  fda_profile_read waits for the recorded events and returns the
 * accumulated kernel time in milliseconds and the number of launches it covers since the
 * last reset.  Events are created on first enable and destroyed with the context.  Leave it off
 * while a stream is being captured into a HIP graph (the entry points themselves can be captured:
 * they allocate nothing and record no memset; make the first call of a context outside the capture,
 * since that one also tabulates the hash).
 */
int fda_profile_enable(fda_ctx* ctx, int on);
int fda_profile_read(fda_ctx* ctx, double* state_kernel_ms, int64_t* launches, int reset);

/*
 * Measurement aids (no part of the method): kernels of known HBM traffic and of known LDS work, so
 * that the rates the FDA kernels are compared with are measured on the same device by the same
 * library.  Both create two HIP events, run one untimed launch, time the rest and wait for `stream`.
 *
 * fda_calib_stream: a pass over `bytes` bytes (rounded down to whole 16-byte vectors, one vector per
 * lane and access, every workgroup on a contiguous range) repeated `reps` times;  mode 0 reads src
 * (dst: DEVICE, 4 bytes, a sink that is practically never written),  mode 1 fills dst (src unused),
 * mode 2 copies src to dst (reads `bytes`, writes `bytes`);  modes 4, 5, 6: the same with the
 * nontemporal hint on every load and store.  src, dst: DEVICE, 16-byte aligned.  *ms_per_rep: HOST,
 * written.
 *
 * fda_calib_lds_atomics: one workgroup of 512 threads per compute unit adds into 144 KiB of LDS cells,
 * `iters` times eight atomic additions per lane to cell addresses fixed at the start.
 *   op       0: 32-bit integer add returning the old value, 1: 32-bit integer add, 2: 64-bit integer
 *            add, 3: fp64 add, 4: fp32 add, 5: 64-bit integer add returning the old value, 6 / 7: no
 *            addition, a plain read of 8 / 16 bytes (the cell moves by a fixed step per iteration)
 *   pattern  0: every lane its own random cell, 1: lane t on cell t (no conflicts), 2/3/4/5: groups of
 *            4/8/16/32 lanes on consecutive cells of a random group
 *   sink_dev DEVICE, 4 bytes (practically never written)
 * *lane_ops_per_clock_per_cu: HOST, additions per lane, per clock of the device's reported clock rate,
 * per compute unit;  *clock_ghz (may be NULL): that clock rate.
 */
int fda_calib_stream(int mode, const void* src, void* dst, size_t bytes, int reps, void* stream,
                     double* ms_per_rep);
int fda_calib_lds_atomics(int op, int pattern, int iters, void* sink_dev, void* stream,
                          double* lane_ops_per_clock_per_cu, double* clock_ghz);

#ifdef __cplusplus
}
#endif
#endif /* FDA_H_ */
