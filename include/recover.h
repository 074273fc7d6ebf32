/*
 * recover.h - C ABI of the ReCoVer data-parallel gradient path on one MI355X (gfx950).
 *
 * One context holds what W_init data-parallel replicas hold for one parameter shard: a flat
 * fp32 gradient accumulator per replica, an optional snapshot per replica, the reduced
 * gradient, and the fp32 optimiser state, all as separate buffers in the memory of ONE GPU.
 * The calls below are the numeric statements of one iteration of the paper's protocol
 * (Alg. 1) with the forward/backward pass replaced by a gradient handed in by the caller:
 *
 *   recover_accumulate     Alg. 1, local accumulation: acc += gradient, dropped once the quota is met
 *   recover_snapshot       Alg. 1, snapshot step (Sec. 4.2): S(b) <- b, tag eps(b) <- eps_cur
 *   recover_reduce         Alg. 2 "Reduce" and the division of Alg. 1's commit step: sum over non-spare
 *                          survivors, then / B
 *   recover_policy_adjust  Alg. 2 "Record", Alg. 4, Alg. 6 (failure set given) or Alg. 7 (empty set)
 *   recover_restore        Alg. 5: stale = {b : eps(b) < eps_cur}; copy S(b) -> b
 *   recover_adamw_step     Alg. 1, commit step: optimiser step; ends the iteration
 *
 * plus one-pass variants that give the same bits as the calls they replace
 * (recover_accumulate_snapshot, recover_accumulate_many, recover_reduce_adamw_step), queries, and a
 * device-side buffer comparison for verification.  Every device call only launches kernels (no
 * allocation, no memset, no host wait), so a sequence of calls can be captured into a HIP graph;
 * see recover_config.step_state for what the optimiser step needs then.
 *
 * Notation is the paper's (Sec. 4.3): W_init replicas, G_init microbatches per replica,
 * B = W_init * G_init microbatches per iteration (constant for the life of a context, Eq. 1),
 * W_cur survivors, G_cur / R_cur the quota of a major / of the minor, eps the world epoch.
 * A "bucket" b is one tensor of the shard: tensor t covers elements
 * [tensor_offsets[t], tensor_offsets[t+1]) of every flat buffer.
 *
 * Memory.  "device" = a pointer into the GPU's memory, "host" = ordinary process memory.
 * Every device buffer is owned by the caller, must stay valid until recover_destroy, must be
 * 16-byte aligned, and is never freed, reallocated or synchronised by the library.  Device
 * work is enqueued on the `hip_stream` argument (a hipStream_t, NULL = the default stream)
 * and the calls return without waiting for it; host bookkeeping is updated at call time, so
 * all calls on one context must come from one thread at a time.  Calls on one context may use
 * different streams: each call's device work is ordered after the previous call's by an event
 * (no host wait), so e.g. recover_restore can run on a side stream while the caller's own
 * kernels keep the main stream busy, and the next recover_accumulate waits for the rewind
 * (the non-blocking restoration of Sec. 4.2).  Work of the CALLER that reads or writes the
 * context's buffers must be ordered by the caller.  recover_policy_adjust and the query calls
 * touch no device memory.
 *
 * Errors.  Every call returns RECOVER_OK (0), RECOVER_SKIPPED (1, nothing enqueued, not an
 * error) or a negative code; nothing throws or aborts.  After any negative return other than
 * RECOVER_ERR_HIP the context is unchanged and nothing was enqueued; after RECOVER_ERR_HIP the
 * device buffers the call writes are undefined.  recover_last_error gives a message.
 * The library has no CPU fallback: without a usable GPU every device call fails with
 * RECOVER_ERR_HIP (except on a context created with RECOVER_FLAG_HOST_ONLY).
 */
#ifndef RECOVER_H
#define RECOVER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct recover_ctx recover_ctx; /* opaque, library-owned, freed by recover_destroy */

enum {
  RECOVER_OK = 0,
  RECOVER_SKIPPED = 1,          /* quota already met (Alg. 1, quota test) or group quiesced (Alg. 2, quiesce test) */
  RECOVER_ERR_ARG = -1,         /* bad pointer, range, replica index, dtype or flag */
  RECOVER_ERR_STATE = -2,       /* call not allowed in the current protocol state */
  RECOVER_ERR_NO_SURVIVOR = -3, /* the failure set would leave no replica (Sec. 4, Claim) */
  RECOVER_ERR_HIP = -4,         /* a HIP runtime call failed */
  RECOVER_ERR_ALIGN = -5,       /* a device pointer is not 16-byte aligned */
  RECOVER_ERR_NO_SNAPSHOT = -6  /* the call needs snapshot buffers and the context was created without */
};

enum { RECOVER_F32 = 0, RECOVER_BF16 = 1 }; /* element type of a microbatch gradient */

enum { /* replica roles (Sec. 4.3) */
  RECOVER_ROLE_MAJOR = 0,
  RECOVER_ROLE_MINOR = 1,
  RECOVER_ROLE_MAJOR_SPARE = 2,
  RECOVER_ROLE_MINOR_SPARE = 3,
  RECOVER_ROLE_DEAD = 4
};

enum { RECOVER_RESTORE_SKIP = 0, RECOVER_RESTORE_BLOCKING = 1, RECOVER_RESTORE_NONBLOCKING = 2 }; /* Alg. 5 */

enum { /* recover_config.flags */
  RECOVER_FLAG_ADAPTIVE = 1u,  /* Alg. 8 strawman instead of the static-world policy: never a boundary,
                                  the batch shrinks with the world, the divisor is the committed count */
  RECOVER_FLAG_ANY_ORDER = 2u, /* do not require ascending microbatch ids inside a replica */
  RECOVER_FLAG_HOST_ONLY = 4u  /* bookkeeping only: no kernel is launched and no device pointer is
                                  touched (they may be NULL); for tests of the host logic */
};

enum { RECOVER_REDUCE_INPLACE = 1u };   /* recover_reduce flags */
enum { RECOVER_FUSED_WRITE_GRAD = 1u }; /* recover_reduce_adamw_step flags */

typedef struct {
  int32_t W_init;                /* replicas, 1..RECOVER_MAX_REPLICAS */
  int32_t G_init;                /* microbatches per replica per iteration, >= 1 */
  int64_t n_elems;               /* elements of the shard = tensor_offsets[n_tensors], 0..RECOVER_MAX_ELEMS */
  int32_t n_tensors;             /* >= 1 */
  const int64_t *tensor_offsets; /* host, n_tensors + 1 non-decreasing element offsets from 0; copied */
  float *const *acc;             /* host array of W_init device pointers, n_elems floats each */
  float *const *snap;            /* host array of W_init device pointers, or NULL (no snapshots); with
                                    RECOVER_FLAG_HOST_ONLY only the presence of the array counts */
  float *grad_out;               /* device, n_elems floats: the iteration gradient */
  float *param;                  /* device, n_elems floats: fp32 master parameters */
  float *exp_avg;                /* device, n_elems floats: AdamW first moment */
  float *exp_avg_sq;             /* device, n_elems floats: AdamW second moment */
  uint16_t *param_bf16;          /* device, n_elems bf16 or NULL: rounded copy of param after each step */
  uint32_t flags;
  void *step_state;              /* device, 64 bytes, zero-filled by the caller before the first step, or NULL.
                                    If given, the optimiser's step count and bias-correction products live
                                    there and advance on the device (a one-thread kernel before each update),
                                    so that a HIP graph captured around an iteration stays correct when it is
                                    replayed; the results are the same bits as without it. */
} recover_config;

#define RECOVER_MAX_REPLICAS 64
/* Largest shard: every kernel launch is one workgroup per 256 elements and a grid holds fewer than 2^31
 * workgroups in x.  All element and byte offsets are 64-bit throughout. */
#define RECOVER_MAX_ELEMS (1ll << 38)

/* The failure record of Alg. 2 "Record" plus the PolicyDecision of Alg. 6 (failure case), or the
 * layout of Alg. 7 (commit case), or the current state (recover_query).  The four arrays are
 * caller-owned host arrays of W_init entries each, or NULL to skip them. */
typedef struct {
  int32_t at_boundary;  /* a vacated slot found no spare of its role */
  int32_t restore_mode; /* RECOVER_RESTORE_* latched for the next recover_restore */
  int32_t epoch;        /* eps_cur after this call */
  int32_t W_cur;        /* survivors, spares included */
  int32_t C_cur;        /* microbatches finished by contributing survivors */
  int32_t G_ext;        /* extra microbatches of a boundary step, else 0 */
  int32_t n_bdry;       /* boundary minors designated by this call */
  int32_t G_cur;
  int32_t R_cur;
  int32_t loop_bound;   /* P(major): microbatch slots of this iteration */
  int32_t n_maj, n_min, n_ms, n_mi, n_bm; /* role census after the call */
  int32_t *role;
  int32_t *target;      /* quota for the whole iteration */
  int32_t *contributed; /* microbatches fully accumulated so far */
  int32_t *is_boundary_minor;
} recover_decision;

/* Create a context.  Roles start as W_init majors at quota G_init, eps = 0, iteration 0 open.
 * ERR_ARG on bad sizes or offsets or a NULL required pointer, ERR_ALIGN on alignment. */
int recover_init(const recover_config *cfg, recover_ctx **out);
int recover_destroy(recover_ctx *ctx);

/* Alg. 1, local accumulation.  acc[replica][i] += widen(grad[i]) for i in tensors [tensor_begin, tensor_end);
 * the first microbatch of a replica in an iteration stores (+0) + widen(grad[i]) instead, which
 * replaces "zero gradients" of Alg. 1, start of the iteration.  `grad` is a device pointer to the FLAT gradient
 * of the whole shard (n_elems elements of `dtype`), indexed like acc.  A microbatch may arrive
 * in several calls over disjoint tensor ranges, all with the same id; it counts as contributed
 * once every tensor has taken it.  Returns SKIPPED when contributed >= target.  ERR_STATE: dead
 * replica, policy advancement pending, tensor already holds this microbatch or an in-place sum,
 * another microbatch still incomplete.  ERR_ARG: id not above the replica's previous id
 * (unless RECOVER_FLAG_ANY_ORDER). */
int recover_accumulate(recover_ctx *ctx, int replica, uint32_t global_mb_id, const void *grad, int dtype,
                       int tensor_begin, int tensor_end, void *hip_stream);

/* recover_accumulate over ALL tensors for n distinct replicas in ONE launch: pair i adds grads[i] (device,
 * flat, `dtype`) as microbatch ids[i] into acc[replicas[i]].  `replicas`, `ids`, `grads`, `status_out` are host
 * arrays of n entries; status_out (or NULL) receives RECOVER_OK or RECOVER_SKIPPED (quota met) per pair.  Every
 * pair is checked as by recover_accumulate before anything is enqueued; on a negative return nothing happened.
 * Returns SKIPPED if every pair was skipped.  Same bits as n separate calls; for shards so small that the
 * launch, not HBM, bounds an accumulate. */
int recover_accumulate_many(recover_ctx *ctx, int n, const int32_t *replicas, const uint32_t *ids,
                            const void *const *grads, int dtype, int32_t *status_out, void *hip_stream);

/* recover_accumulate followed by recover_snapshot of the same replica and tensor range in ONE pass: the
 * new accumulator value is stored to acc and to snap (Alg. 1: local accumulation and snapshot in one pass; 4 bytes per element
 * less than the two calls).  Same results, bookkeeping and errors as the two calls; ERR_NO_SNAPSHOT
 * without snapshot buffers.  For callers that snapshot at every microbatch boundary. */
int recover_accumulate_snapshot(recover_ctx *ctx, int replica, uint32_t global_mb_id, const void *grad, int dtype,
                                int tensor_begin, int tensor_end, void *hip_stream);

/* Alg. 1, snapshot step, Sec. 4.2.  snap[r][range] <- acc[r][range]; records (eps_cur, microbatch
 * count) per (replica, tensor).  replica = -1: every survivor. */
int recover_snapshot(recover_ctx *ctx, int replica, int tensor_begin, int tensor_end, void *hip_stream);

/* Alg. 5.  For every snapshotted tensor of the replica (-1: every survivor) that is stale
 * (tag < eps_cur), or every snapshotted tensor if stale_only == 0: acc <- snap, microbatch count
 * <- the snapshot's, so work accumulated after the snapshot is as if never accumulated.  Lifts
 * the quiesce; in NON-BLOCKING mode the replica's snapshot records are then cleared (the extended
 * pass takes fresh ones).  ERR_STATE if the rewind would leave a replica's tensors at different
 * microbatch counts (nothing is copied then).  On a context without snapshot buffers nothing was
 * ever snapshotted, so the stale set is empty (Alg. 5, SKIP): the call only lifts the quiesce, and
 * returns ERR_NO_SNAPSHOT if a bucket holds an in-place sum that it cannot take back. */
int recover_restore(recover_ctx *ctx, int replica, int stale_only, void *hip_stream);

/* n_failed > 0: Alg. 2 "Record" + Alg. 4 + Alg. 6 for the failure set failed[0..n_failed)
 * (original replica indices): survivors shrink, eps += 1, vacated slots are filled from spares of
 * the same role, else a policy boundary extends the quotas so that they sum to B again; later
 * reductions are quiesced until recover_restore.  n_failed == 0: Alg. 7, the steady-state layout
 * after an iteration that crossed a boundary (no-op otherwise); must be called after
 * recover_adamw_step of such an iteration before the next accumulate.  Host only. */
int recover_policy_adjust(recover_ctx *ctx, const int32_t *failed, int n_failed, recover_decision *out);

/* Alg. 2 "Reduce" and the division of Alg. 1, commit step.  For tensors [tensor_begin, tensor_end):
 * grad_out[i] = (sum over contributing survivors r, ascending, of acc[r][i]) / B, contributors =
 * majors and minors that hold at least one microbatch in that tensor.  RECOVER_REDUCE_INPLACE also
 * leaves the undivided sum in every survivor's acc (what an all-reduce does; needed to model a
 * failure during synchronisation).  SKIPPED while quiesced. */
int recover_reduce(recover_ctx *ctx, int tensor_begin, int tensor_end, uint32_t flags, void *hip_stream);

/* Alg. 1, commit step.  Decoupled-weight-decay Adam on (param, exp_avg, exp_avg_sq) with grad_out, step
 * count kept by the context (from 1).  ERR_STATE unless every tensor was reduced under the current
 * epoch, is unchanged since, and holds exactly B microbatches (Eq. 1).  Ends the iteration:
 * counters, quotas, snapshot records and boundary-minor marks are reset. */
int recover_adamw_step(recover_ctx *ctx, float lr, float beta1, float beta2, float eps, float weight_decay,
                       void *hip_stream);

/* recover_adamw_step for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc) and still want the step count to live on the device:
 * the 64-byte step state that recover_config.step_state otherwise brings in is slot `slot` of an array of
 * RECOVER_STATIC_STEP_SLOTS states that the library keeps in a file-scope device array (4 KiB on every GPU
 * the library runs on, held until the process ends; the slot of the CURRENT device is used).  restart != 0:
 * the slot is cleared first (by a kernel, not a memset), so this is step 1; otherwise the slot's count goes on
 * from the last call that used it, whichever context made it: a slot belongs to one context at a time, the
 * caller assigns the slots, and calls that use one slot from several streams or threads at once race.
 * Allocates nothing.  ERR_ARG: slot outside [0, RECOVER_STATIC_STEP_SLOTS).  ERR_STATE: the context has a
 * caller-owned step state; otherwise as recover_adamw_step, with the same bits in param, exp_avg, exp_avg_sq. */
#define RECOVER_STATIC_STEP_SLOTS 64
int recover_adamw_step_static(recover_ctx *ctx, int slot, int restart, float lr, float beta1, float beta2, float eps,
                              float weight_decay, void *hip_stream);

/* recover_reduce over all tensors (not in place) followed by recover_adamw_step, in ONE pass over the
 * contributors' buffers and the optimiser state: 4 R_c + 24 bytes per element instead of 4 R_c + 32.  grad_out
 * holds the gradient after the call only with RECOVER_FUSED_WRITE_GRAD (without the flag its content is
 * unspecified).  Where more than RECOVER_TUNE_ONE_PASS_MAX contributors (default 32) hold a tensor the call
 * launches the reduction and then the update for it instead, which is faster there.  Same checks (Eq. 1), same
 * bits in param, exp_avg, exp_avg_sq (and grad_out if asked for) as the two calls.  Ends the iteration. */
int recover_reduce_adamw_step(recover_ctx *ctx, float lr, float beta1, float beta2, float eps, float weight_decay,
                              uint32_t flags, void *hip_stream);

/* Current state in the layout of a decision (at_boundary = a boundary was crossed this iteration). */
int recover_query(recover_ctx *ctx, recover_decision *out);

/* Audit: ids of the microbatches fully accumulated into acc[replica] this iteration, in order.
 * Writes min(count, cap) ids and returns the count, or a negative code. */
int recover_committed_ids(recover_ctx *ctx, int replica, uint32_t *ids_out, int cap);

/* Verification support (not a step of the path): compares two device fp32 buffers (16-byte aligned) of n elements on the GPU.
 * The 40-byte result is written to DEVICE memory `out_device` (caller-owned, 8-byte aligned), asynchronously on
 * the stream; the caller copies it back.  max_abs_diff and max_abs_ref skip NaNs; the checksums are
 * sum(bits[i] * (2 i + 1)) mod 2^64, so equal checksums of x and ref with n_mismatch == 0 mean equal buffers.
 * The result does not depend on the launch shape. */
typedef struct {
  uint64_t n_mismatch;   /* elements whose bit patterns differ */
  uint64_t n_nan;        /* elements where x or ref is a NaN */
  uint64_t checksum_x;
  uint64_t checksum_ref;
  float max_abs_diff;    /* max |x[i] - ref[i]| */
  float max_abs_ref;     /* max |ref[i]| */
} recover_compare_result;
int recover_compare(const float *x, const float *ref, int64_t n, recover_compare_result *out_device, void *hip_stream);

/* Allocation helpers for callers that want the buffers of a context in ONE device allocation with a fixed relative
 * placement (the context calls themselves never allocate).  recover_device_alloc gives `bytes` of device memory on
 * the current device, 2 MiB-aligned; contiguous != 0 asks the driver for physically contiguous memory
 * (hipDeviceMallocContiguous), which keeps the translation fragments large, and fails with ERR_HIP if the driver cannot
 * provide it (the caller then allocates normally).  The memory is not cleared.  recover_device_free releases it; the
 * caller makes sure no work that uses it is in flight.
 * Placement note (measured on MI355X): the streams of one kernel launch (a gradient and the accumulator it is added to;
 * the reduced gradient and the optimiser state; the accumulators of one reduction) run up to 7 % faster together when
 * they lie in the same zone of physical memory; inside a large physically contiguous allocation the zones end at
 * multiples of 32 GiB from its start.  So carve buffers that stream together from one such window, next to each other;
 * buffers of different groups (snapshots, another replica's pair) can go to other windows. */
int recover_device_alloc(uint64_t bytes, int contiguous, void **out_device);
int recover_device_free(void *device);

/* Message of the last negative return on this context (or of recover_init if ctx == NULL). */
const char *recover_last_error(const recover_ctx *ctx);

/* Launch-shape knobs, for measurement sweeps only.  They are PROCESS-GLOBAL (shared by every context) and not
 * thread-safe: set them while no other thread is inside the library.  The results never depend on them.  Values
 * outside the documented sets are rejected with ERR_ARG and change nothing. */
enum { /* kernel classes that have a launch shape of their own */
  RECOVER_KERNEL_ACCUMULATE_FIRST_F32 = 0, /* first microbatch of a replica: no read of acc */
  RECOVER_KERNEL_ACCUMULATE_RMW_F32 = 1,
  RECOVER_KERNEL_ACCUMULATE_FIRST_BF16 = 2,
  RECOVER_KERNEL_ACCUMULATE_RMW_BF16 = 3,
  RECOVER_KERNEL_COPY = 4, /* snapshot and restore */
  RECOVER_KERNEL_REDUCE = 5,
  RECOVER_KERNEL_ADAMW = 6,
  RECOVER_KERNEL_REDUCE_ADAMW = 7,
  RECOVER_KERNEL_ACCUMULATE_SNAPSHOT_F32 = 8,  /* recover_accumulate_snapshot: the dual store */
  RECOVER_KERNEL_ACCUMULATE_SNAPSHOT_BF16 = 9,
  RECOVER_KERNEL_CLASSES = 10
};
enum { /* keys of recover_set_tuning / recover_get_tuning */
  RECOVER_TUNE_NONTEMPORAL = 1, /* {0, 1}: streaming cache hints on loads and stores */
  RECOVER_TUNE_ONE_PASS_MAX = 2, /* 0..RECOVER_MAX_REPLICAS: most contributors for which recover_reduce_adamw_step
                                    runs as one kernel; with more it launches the reduction, then the update */
  RECOVER_TUNE_THREADS = 7,     /* {64, 256}: lanes per workgroup */
  RECOVER_TUNE_VECS = 16,       /* + kernel class: 128-bit vectors per lane per stream {1, 2, 4} */
  RECOVER_TUNE_WAVES = 32,      /* + kernel class: wavefronts resident per CU, 0 = hardware limit, else 2..32 */
  RECOVER_TUNE_DEPTH = 48       /* + RECOVER_KERNEL_REDUCE or _REDUCE_ADAMW: contributors a wavefront loads at a time {1, 2} */
};
int recover_set_tuning(int key, int value);
int recover_get_tuning(int key, int *value);

#ifdef __cplusplus
}
#endif
#endif /* RECOVER_H */
