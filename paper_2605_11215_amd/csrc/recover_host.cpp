// Host side of the C ABI declared in include/recover.h: argument checks, the integer
// versatile-workload policy (Sec. 4.3; Alg. 2 "Record", Alg. 4, 6, 7, 8), the per-bucket
// bookkeeping of Sec. 4.2 (snapshot + world-epoch tag, stale set of Alg. 5), and the launches of
// the kernels in kernels.hip.  No arithmetic on gradient data happens here.
#include "../../include/recover.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "kernels.h"

using recover::kMaxReplicas;
static_assert(RECOVER_STATIC_STEP_SLOTS == recover::kStaticStepSlots, "slot counts of the header and of the kernels must agree");
static_assert(RECOVER_KERNEL_CLASSES == recover::kNumClasses, "kernel classes of the header and of the launchers must agree");

struct recover_ctx {
  int W = 0, G = 0, B = 0, T = 0;
  int64_t N = 0;
  std::vector<int64_t> off;
  float *acc[kMaxReplicas] = {};
  float *snap[kMaxReplicas] = {};
  bool have_snap = false;
  float *grad_out = nullptr, *param = nullptr, *exp_avg = nullptr, *exp_avg_sq = nullptr;
  uint16_t *param_bf16 = nullptr;
  bool adaptive = false, any_order = false, host_only = false;

  // policy state (Sec. 4.3)
  int role[kMaxReplicas] = {};
  int target[kMaxReplicas] = {};
  int contributed[kMaxReplicas] = {};
  bool bdry_minor[kMaxReplicas] = {};
  int G_cur = 0, R_cur = 0, eps = 0, loop_bound = 0;
  bool crossed_boundary = false, pending_advance = false, quiesced = false;
  int restore_mode = RECOVER_RESTORE_SKIP;

  // bucket bookkeeping (Sec. 4.2), index r * T + b
  std::vector<int> cnt, snap_cnt, snap_eps;
  std::vector<uint8_t> snap_valid, holds_sum;
  // per tensor: the last reduction
  std::vector<int> red_eps, red_total;
  std::vector<uint8_t> red_dirty;
  // audit of accumulated microbatch ids
  std::vector<uint32_t> ids[kMaxReplicas];
  bool open_mb[kMaxReplicas] = {};
  uint32_t open_id[kMaxReplicas] = {};

  long step = 0;  // optimiser steps taken
  double beta1_pow = 1.0, beta2_pow = 1.0;      // running products beta^t of the steps taken
  recover::StepState *step_state = nullptr;     // optional device-resident step state
  std::string err;

  // Stream ordering: device calls on one context may come on different streams (the rewind of
  // Alg. 5 runs on a side stream); each call is ordered after the previous one with an event.
  hipStream_t last_stream = nullptr;
  bool have_last_stream = false;
  hipEvent_t order_event = nullptr;
};

static std::string g_init_err;

static int fail(recover_ctx *c, int code, const char *fmt, ...) {
  char buf[256];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c)
    c->err = buf;
  else
    g_init_err = buf;
  return code;
}

static inline bool alive(const recover_ctx *c, int r) { return c->role[r] != RECOVER_ROLE_DEAD; }
static inline bool contributor(const recover_ctx *c, int r) {
  return c->role[r] == RECOVER_ROLE_MAJOR || c->role[r] == RECOVER_ROLE_MINOR;
}
static int quota_of(const recover_ctx *c, int role) {
  if (role == RECOVER_ROLE_MAJOR || role == RECOVER_ROLE_MAJOR_SPARE) return c->G_cur;
  if (role == RECOVER_ROLE_MINOR || role == RECOVER_ROLE_MINOR_SPARE) return c->R_cur;
  return 0;
}
static int count_alive(const recover_ctx *c) {
  int n = 0;
  for (int r = 0; r < c->W; ++r) n += alive(c, r);
  return n;
}
static int finished_by_contributors(const recover_ctx *c) {
  int n = 0;
  for (int r = 0; r < c->W; ++r)
    if (contributor(c, r)) n += c->contributed[r];
  return n;
}

// Quotas and counters of a new iteration from the role layout in force (Sec. 4.3).
static void prime_quotas(recover_ctx *c) {
  for (int r = 0; r < c->W; ++r) {
    c->contributed[r] = 0;
    c->target[r] = quota_of(c, c->role[r]);
    c->bdry_minor[r] = false;
  }
  c->loop_bound = c->G_cur;
  c->crossed_boundary = false;
  c->restore_mode = RECOVER_RESTORE_SKIP;
}

// Alg. 1, start of the iteration: counters to zero, quotas from the roles, bookkeeping cleared.
static void open_iteration(recover_ctx *c) {
  prime_quotas(c);
  for (int r = 0; r < c->W; ++r) {
    c->ids[r].clear();
    c->open_mb[r] = false;
  }
  c->quiesced = false;
  std::fill(c->cnt.begin(), c->cnt.end(), 0);
  std::fill(c->snap_valid.begin(), c->snap_valid.end(), 0);
  std::fill(c->holds_sum.begin(), c->holds_sum.end(), 0);
  std::fill(c->red_eps.begin(), c->red_eps.end(), -1);
  std::fill(c->red_total.begin(), c->red_total.end(), 0);
  std::fill(c->red_dirty.begin(), c->red_dirty.end(), 1);
}

static void fill_decision(const recover_ctx *c, recover_decision *d, bool at_boundary, int G_ext, int n_bdry) {
  if (!d) return;
  d->at_boundary = at_boundary;
  d->restore_mode = c->restore_mode;
  d->epoch = c->eps;
  d->W_cur = count_alive(c);
  d->C_cur = finished_by_contributors(c);
  d->G_ext = G_ext;
  d->n_bdry = n_bdry;
  d->G_cur = c->G_cur;
  d->R_cur = c->R_cur;
  d->loop_bound = c->loop_bound;
  d->n_maj = d->n_min = d->n_ms = d->n_mi = d->n_bm = 0;
  for (int r = 0; r < c->W; ++r) {
    if (!alive(c, r)) continue;
    if (c->bdry_minor[r]) {
      d->n_bm++;
      continue;
    }
    switch (c->role[r]) {
      case RECOVER_ROLE_MAJOR: d->n_maj++; break;
      case RECOVER_ROLE_MINOR: d->n_min++; break;
      case RECOVER_ROLE_MAJOR_SPARE: d->n_ms++; break;
      case RECOVER_ROLE_MINOR_SPARE: d->n_mi++; break;
    }
  }
  for (int r = 0; r < c->W; ++r) {
    if (d->role) d->role[r] = c->role[r];
    if (d->target) d->target[r] = c->target[r];
    if (d->contributed) d->contributed[r] = c->contributed[r];
    if (d->is_boundary_minor) d->is_boundary_minor[r] = c->bdry_minor[r];
  }
}

// Orders the work about to be enqueued on `s` after the context's previous device call if that
// call used another stream: record an event there, make `s` wait for it.  No host wait.
// While `s` is being captured into a graph, streams outside the capture must not be touched (the
// runtime would invalidate the capture): the wait is then inserted only if the previous stream
// belongs to a capture too (a fork inside the same graph); whoever starts a capture has made
// earlier work finish, as graph capture requires anyway.
static int order_after_previous(recover_ctx *c, hipStream_t s, const char *who) {
  if (c->host_only) return RECOVER_OK;
  hipStreamCaptureStatus now = hipStreamCaptureStatusNone;
  if (s != nullptr && hipStreamIsCapturing(s, &now) != hipSuccess) now = hipStreamCaptureStatusNone;
  const bool capturing = now == hipStreamCaptureStatusActive;
  if (c->have_last_stream && c->last_stream != s) {
    bool insert = true;
    if (capturing) {
      hipStreamCaptureStatus prev = hipStreamCaptureStatusNone;
      insert = c->last_stream != nullptr && hipStreamIsCapturing(c->last_stream, &prev) == hipSuccess &&
               prev == hipStreamCaptureStatusActive;
    }
    if (insert) {
      hipError_t he = hipSuccess;
      if (!c->order_event) he = hipEventCreateWithFlags(&c->order_event, hipEventDisableTiming);
      if (he == hipSuccess) he = hipEventRecord(c->order_event, c->last_stream);
      if (he == hipSuccess) he = hipStreamWaitEvent(s, c->order_event, 0);
      if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "%s: stream ordering: %s", who, hipGetErrorString(he));
    }
  }
  c->last_stream = s;
  c->have_last_stream = true;
  return RECOVER_OK;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" {

int recover_init(const recover_config *cfg, recover_ctx **out) {
  if (!cfg || !out) return fail(nullptr, RECOVER_ERR_ARG, "recover_init: NULL argument");
  *out = nullptr;
  if (cfg->W_init < 1 || cfg->W_init > kMaxReplicas || cfg->G_init < 1)
    return fail(nullptr, RECOVER_ERR_ARG, "recover_init: W_init must be 1..%d and G_init >= 1", kMaxReplicas);
  if ((int64_t)cfg->W_init * cfg->G_init > (1 << 24))
    return fail(nullptr, RECOVER_ERR_ARG, "recover_init: B = W_init * G_init too large");
  if (cfg->n_tensors < 1 || !cfg->tensor_offsets || cfg->n_elems < 0)
    return fail(nullptr, RECOVER_ERR_ARG, "recover_init: tensor table missing");
  if (cfg->n_elems > RECOVER_MAX_ELEMS)
    return fail(nullptr, RECOVER_ERR_ARG, "recover_init: n_elems above RECOVER_MAX_ELEMS (2^38)");
  if (cfg->flags & ~(RECOVER_FLAG_ADAPTIVE | RECOVER_FLAG_ANY_ORDER | RECOVER_FLAG_HOST_ONLY))
    return fail(nullptr, RECOVER_ERR_ARG, "recover_init: unknown flag");
  if (cfg->tensor_offsets[0] != 0 || cfg->tensor_offsets[cfg->n_tensors] != cfg->n_elems)
    return fail(nullptr, RECOVER_ERR_ARG, "recover_init: offsets must run from 0 to n_elems");
  for (int t = 0; t < cfg->n_tensors; ++t)
    if (cfg->tensor_offsets[t] > cfg->tensor_offsets[t + 1])
      return fail(nullptr, RECOVER_ERR_ARG, "recover_init: offsets must not decrease");
  const bool host_only = cfg->flags & RECOVER_FLAG_HOST_ONLY;
  if (!host_only) {
    if (!cfg->acc || !cfg->grad_out || !cfg->param || !cfg->exp_avg || !cfg->exp_avg_sq)
      return fail(nullptr, RECOVER_ERR_ARG, "recover_init: NULL device buffer");
    const void *one[] = {cfg->grad_out, cfg->param, cfg->exp_avg, cfg->exp_avg_sq, cfg->param_bf16, cfg->step_state};
    for (const void *p : one)
      if (!aligned16(p)) return fail(nullptr, RECOVER_ERR_ALIGN, "recover_init: buffer not 16-byte aligned");
    for (int r = 0; r < cfg->W_init; ++r) {
      if (!cfg->acc[r] || (cfg->snap && !cfg->snap[r]))
        return fail(nullptr, RECOVER_ERR_ARG, "recover_init: NULL replica buffer %d", r);
      if (!aligned16(cfg->acc[r]) || (cfg->snap && !aligned16(cfg->snap[r])))
        return fail(nullptr, RECOVER_ERR_ALIGN, "recover_init: replica buffer %d not 16-byte aligned", r);
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1)
      return fail(nullptr, RECOVER_ERR_HIP, "recover_init: no usable GPU (this library has no CPU path)");
  }
  recover_ctx *c = new recover_ctx();
  c->W = cfg->W_init;
  c->G = cfg->G_init;
  c->B = cfg->W_init * cfg->G_init;
  c->T = cfg->n_tensors;
  c->N = cfg->n_elems;
  c->off.assign(cfg->tensor_offsets, cfg->tensor_offsets + cfg->n_tensors + 1);
  c->host_only = host_only;
  c->adaptive = cfg->flags & RECOVER_FLAG_ADAPTIVE;
  c->any_order = cfg->flags & RECOVER_FLAG_ANY_ORDER;
  c->have_snap = cfg->snap != nullptr;  // host-only: the array's entries may be NULL, its presence counts
  if (!host_only) {
    for (int r = 0; r < c->W; ++r) {
      c->acc[r] = cfg->acc[r];
      c->snap[r] = cfg->snap ? cfg->snap[r] : nullptr;
    }
    c->grad_out = cfg->grad_out;
    c->param = cfg->param;
    c->exp_avg = cfg->exp_avg;
    c->exp_avg_sq = cfg->exp_avg_sq;
    c->param_bf16 = cfg->param_bf16;
    c->step_state = reinterpret_cast<recover::StepState *>(cfg->step_state);
  }
  for (int r = 0; r < c->W; ++r) c->role[r] = RECOVER_ROLE_MAJOR;
  c->G_cur = c->G;
  c->R_cur = 0;
  const size_t wt = (size_t)c->W * c->T;
  c->cnt.assign(wt, 0);
  c->snap_cnt.assign(wt, 0);
  c->snap_eps.assign(wt, 0);
  c->snap_valid.assign(wt, 0);
  c->holds_sum.assign(wt, 0);
  c->red_eps.assign(c->T, -1);
  c->red_total.assign(c->T, 0);
  c->red_dirty.assign(c->T, 1);
  open_iteration(c);
  *out = c;
  return RECOVER_OK;
}

int recover_destroy(recover_ctx *c) {
  if (c && c->order_event) (void)hipEventDestroy(c->order_event);
  delete c;
  return RECOVER_OK;
}

const char *recover_last_error(const recover_ctx *c) { return c ? c->err.c_str() : g_init_err.c_str(); }

static int check_range(recover_ctx *c, int tb, int te, const char *who) {
  if (tb < 0 || te > c->T || tb > te) return fail(c, RECOVER_ERR_ARG, "%s: tensor range [%d, %d) outside [0, %d)", who, tb, te, c->T);
  return RECOVER_OK;
}

static int accumulate_impl(recover_ctx *c, int r, uint32_t mb_id, const void *grad, int dtype, int tb, int te,
                           void *stream, bool with_snapshot) {
  if (!c) return RECOVER_ERR_ARG;
  if (r < 0 || r >= c->W) return fail(c, RECOVER_ERR_ARG, "accumulate: replica %d out of range", r);
  if (dtype != RECOVER_F32 && dtype != RECOVER_BF16) return fail(c, RECOVER_ERR_ARG, "accumulate: dtype %d", dtype);
  if (int e = check_range(c, tb, te, "accumulate")) return e;
  if (!c->host_only) {
    if (!grad) return fail(c, RECOVER_ERR_ARG, "accumulate: NULL gradient");
    if (!aligned16(grad)) return fail(c, RECOVER_ERR_ALIGN, "accumulate: gradient not 16-byte aligned");
  }
  if (with_snapshot && !c->have_snap)
    return fail(c, RECOVER_ERR_NO_SNAPSHOT, "accumulate_snapshot: context has no snapshot buffers");
  if (c->pending_advance) return fail(c, RECOVER_ERR_STATE, "accumulate: policy advancement pending (Alg. 7)");
  if (!alive(c, r)) return fail(c, RECOVER_ERR_STATE, "accumulate: replica %d is dead", r);
  if (c->contributed[r] >= c->target[r]) return RECOVER_SKIPPED;
  const int k = c->contributed[r];
  if (c->open_mb[r]) {
    if (c->open_id[r] != mb_id)
      return fail(c, RECOVER_ERR_STATE, "accumulate: microbatch %u of replica %d is incomplete", c->open_id[r], r);
  } else if (!c->any_order && !c->ids[r].empty() && mb_id <= c->ids[r].back()) {
    return fail(c, RECOVER_ERR_ARG, "accumulate: id %u does not ascend within replica %d", mb_id, r);
  }
  int *cnt = &c->cnt[(size_t)r * c->T];
  const uint8_t *sum = &c->holds_sum[(size_t)r * c->T];
  for (int b = tb; b < te; ++b)
    if (cnt[b] != k || sum[b])
      return fail(c, RECOVER_ERR_STATE, "accumulate: tensor %d of replica %d cannot take this microbatch", b, r);
  if (int e = order_after_previous(c, (hipStream_t)stream, "accumulate")) return e;
  if (!c->host_only) {
    hipError_t he = recover::launch_accumulate(c->acc[r], with_snapshot ? c->snap[r] : nullptr, grad,
                                               dtype == RECOVER_BF16, k == 0, (size_t)c->off[tb], (size_t)c->off[te],
                                               (hipStream_t)stream);
    if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "accumulate: %s", hipGetErrorString(he));
  }
  for (int b = tb; b < te; ++b) {
    cnt[b] = k + 1;
    c->red_dirty[b] = 1;
  }
  c->open_mb[r] = true;
  c->open_id[r] = mb_id;
  bool complete = true;
  for (int b = 0; b < c->T; ++b) complete = complete && cnt[b] == k + 1;
  if (complete) {
    c->ids[r].push_back(mb_id);
    c->open_mb[r] = false;
    c->contributed[r] = k + 1;
  }
  if (with_snapshot) {
    for (int b = tb; b < te; ++b) {
      const size_t i = (size_t)r * c->T + b;
      c->snap_valid[i] = 1;
      c->snap_eps[i] = c->eps;
      c->snap_cnt[i] = c->cnt[i];
    }
  }
  return RECOVER_OK;
}

int recover_accumulate(recover_ctx *c, int r, uint32_t mb_id, const void *grad, int dtype, int tb, int te,
                       void *stream) {
  return accumulate_impl(c, r, mb_id, grad, dtype, tb, te, stream, false);
}

int recover_accumulate_many(recover_ctx *c, int n, const int32_t *replicas, const uint32_t *ids,
                            const void *const *grads, int dtype, int32_t *status_out, void *stream) {
  if (!c) return RECOVER_ERR_ARG;
  if (n < 1 || n > c->W || !replicas || !ids || (!c->host_only && !grads))
    return fail(c, RECOVER_ERR_ARG, "accumulate_many: bad argument");
  if (dtype != RECOVER_F32 && dtype != RECOVER_BF16) return fail(c, RECOVER_ERR_ARG, "accumulate_many: dtype %d", dtype);
  if (c->pending_advance) return fail(c, RECOVER_ERR_STATE, "accumulate_many: policy advancement pending (Alg. 7)");
  bool seen[kMaxReplicas] = {};
  for (int i = 0; i < n; ++i) {  // every pair is checked before anything changes
    const int r = replicas[i];
    if (r < 0 || r >= c->W || seen[r]) return fail(c, RECOVER_ERR_ARG, "accumulate_many: replica %d out of range or repeated", r);
    seen[r] = true;
    if (!c->host_only) {
      if (!grads[i]) return fail(c, RECOVER_ERR_ARG, "accumulate_many: NULL gradient");
      if (!aligned16(grads[i])) return fail(c, RECOVER_ERR_ALIGN, "accumulate_many: gradient not 16-byte aligned");
    }
    if (!alive(c, r)) return fail(c, RECOVER_ERR_STATE, "accumulate_many: replica %d is dead", r);
    if (c->contributed[r] >= c->target[r]) continue;
    if (c->open_mb[r])
      return fail(c, RECOVER_ERR_STATE, "accumulate_many: microbatch %u of replica %d is incomplete", c->open_id[r], r);
    if (!c->any_order && !c->ids[r].empty() && ids[i] <= c->ids[r].back())
      return fail(c, RECOVER_ERR_ARG, "accumulate_many: id %u does not ascend within replica %d", ids[i], r);
    for (int b = 0; b < c->T; ++b)
      if (c->cnt[(size_t)r * c->T + b] != c->contributed[r] || c->holds_sum[(size_t)r * c->T + b])
        return fail(c, RECOVER_ERR_STATE, "accumulate_many: tensor %d of replica %d cannot take this microbatch", b, r);
  }
  recover::AccumulateManyArgs a;
  int m = 0, taken[kMaxReplicas];
  for (int i = 0; i < n; ++i) {
    const int r = replicas[i];
    const bool skip = c->contributed[r] >= c->target[r];
    if (status_out) status_out[i] = skip ? RECOVER_SKIPPED : RECOVER_OK;
    if (skip) continue;
    a.acc[m] = c->acc[r];
    a.grad[m] = c->host_only ? nullptr : grads[i];
    a.first[m] = c->contributed[r] == 0;
    taken[m++] = i;
  }
  if (m == 0) return RECOVER_SKIPPED;
  if (int e = order_after_previous(c, (hipStream_t)stream, "accumulate_many")) return e;
  if (!c->host_only) {
    hipError_t he = recover::launch_accumulate_many(a, m, dtype == RECOVER_BF16, 0, (size_t)c->N, (hipStream_t)stream);
    if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "accumulate_many: %s", hipGetErrorString(he));
  }
  for (int j = 0; j < m; ++j) {
    const int r = replicas[taken[j]];
    const int k = c->contributed[r];
    for (int b = 0; b < c->T; ++b) {
      c->cnt[(size_t)r * c->T + b] = k + 1;
      c->red_dirty[b] = 1;
    }
    c->ids[r].push_back(ids[taken[j]]);
    c->contributed[r] = k + 1;
  }
  return RECOVER_OK;
}

int recover_accumulate_snapshot(recover_ctx *c, int r, uint32_t mb_id, const void *grad, int dtype, int tb, int te,
                                void *stream) {
  return accumulate_impl(c, r, mb_id, grad, dtype, tb, te, stream, true);
}

int recover_snapshot(recover_ctx *c, int replica, int tb, int te, void *stream) {
  if (!c) return RECOVER_ERR_ARG;
  if (replica < -1 || replica >= c->W) return fail(c, RECOVER_ERR_ARG, "snapshot: replica %d out of range", replica);
  if (int e = check_range(c, tb, te, "snapshot")) return e;
  if (!c->have_snap) return fail(c, RECOVER_ERR_NO_SNAPSHOT, "snapshot: context has no snapshot buffers");
  if (replica >= 0 && !alive(c, replica)) return fail(c, RECOVER_ERR_STATE, "snapshot: replica %d is dead", replica);
  for (int r = 0; r < c->W; ++r) {
    if ((replica >= 0 && r != replica) || !alive(c, r)) continue;
    for (int b = tb; b < te; ++b)
      if (c->holds_sum[(size_t)r * c->T + b])
        return fail(c, RECOVER_ERR_STATE, "snapshot: tensor %d of replica %d already holds a reduced sum", b, r);
  }
  if (int e = order_after_previous(c, (hipStream_t)stream, "snapshot")) return e;
  recover::CopyManyArgs a;
  int n = 0;
  for (int r = 0; r < c->W; ++r) {
    if ((replica >= 0 && r != replica) || !alive(c, r)) continue;
    a.dst[n] = c->snap[r];
    a.src[n] = c->acc[r];
    ++n;
  }
  if (!c->host_only) {  // one launch whatever the number of replicas
    hipError_t he = n == 1 ? recover::launch_copy(a.dst[0], a.src[0], (size_t)c->off[tb], (size_t)c->off[te], false, (hipStream_t)stream)
                           : recover::launch_copy_many(a, n, (size_t)c->off[tb], (size_t)c->off[te], false, (hipStream_t)stream);
    if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "snapshot: %s", hipGetErrorString(he));
  }
  for (int r = 0; r < c->W; ++r) {
    if ((replica >= 0 && r != replica) || !alive(c, r)) continue;
    for (int b = tb; b < te; ++b) {
      const size_t i = (size_t)r * c->T + b;
      c->snap_valid[i] = 1;
      c->snap_eps[i] = c->eps;
      c->snap_cnt[i] = c->cnt[i];
    }
  }
  return RECOVER_OK;
}

int recover_restore(recover_ctx *c, int replica, int stale_only, void *stream) {
  if (!c) return RECOVER_ERR_ARG;
  if (replica < -1 || replica >= c->W) return fail(c, RECOVER_ERR_ARG, "restore: replica %d out of range", replica);
  if (replica >= 0 && !alive(c, replica)) return fail(c, RECOVER_ERR_STATE, "restore: replica %d is dead", replica);
  if (!c->have_snap) {
    // Without snapshot buffers no bucket was ever snapshotted, so the stale set of Alg. 5 is empty (SKIP):
    // nothing is copied and the quiesce is lifted.  Only a bucket that holds an in-place sum of the old
    // membership cannot be repaired then.
    for (int r = 0; r < c->W; ++r) {
      if ((replica >= 0 && r != replica) || !alive(c, r)) continue;
      for (int b = 0; b < c->T; ++b)
        if (c->holds_sum[(size_t)r * c->T + b])
          return fail(c, RECOVER_ERR_NO_SNAPSHOT, "restore: tensor %d of replica %d holds a reduced sum and the context has no snapshot buffers", b, r);
    }
    c->quiesced = false;
    if (replica < 0) c->restore_mode = RECOVER_RESTORE_SKIP;
    return RECOVER_OK;
  }
  // plan first: which tensors rewind, and whether each replica ends on one microbatch count
  std::vector<uint8_t> pick((size_t)c->W * c->T, 0);
  for (int r = 0; r < c->W; ++r) {
    if ((replica >= 0 && r != replica) || !alive(c, r)) continue;
    int after0 = -1;
    bool any = false, even = true;
    for (int b = 0; b < c->T; ++b) {
      const size_t i = (size_t)r * c->T + b;
      const bool p = c->snap_valid[i] && (!stale_only || c->snap_eps[i] < c->eps);
      pick[i] = p;
      any = any || p;
      const int after = p ? c->snap_cnt[i] : c->cnt[i];
      if (after0 < 0) after0 = after;
      even = even && after == after0;
    }
    if (any && !even)
      return fail(c, RECOVER_ERR_STATE, "restore: rewind would leave replica %d between microbatches", r);
  }
  if (int e = order_after_previous(c, (hipStream_t)stream, "restore")) return e;
  // Device work first.  Replicas that rewind the same set of tensors (the usual case: the buckets that were
  // all-reduced before the failure showed) share one launch per run of adjacent tensors.
  if (!c->host_only) {
    std::vector<uint8_t> done(c->W, 0);
    for (int r0 = 0; r0 < c->W; ++r0) {
      if (done[r0] || (replica >= 0 && r0 != replica) || !alive(c, r0)) continue;
      recover::CopyManyArgs a;
      int n = 0;
      for (int r = r0; r < c->W; ++r) {
        if (done[r] || (replica >= 0 && r != replica) || !alive(c, r)) continue;
        if (memcmp(&pick[(size_t)r * c->T], &pick[(size_t)r0 * c->T], (size_t)c->T) != 0) continue;
        done[r] = 1;
        a.dst[n] = c->acc[r];
        a.src[n] = c->snap[r];
        ++n;
      }
      const uint8_t *pk = &pick[(size_t)r0 * c->T];
      for (int b = 0; b < c->T;) {
        if (!pk[b]) {
          ++b;
          continue;
        }
        int e = b;
        while (e < c->T && pk[e]) ++e;
        hipError_t he = n == 1 ? recover::launch_copy(a.dst[0], a.src[0], (size_t)c->off[b], (size_t)c->off[e], true, (hipStream_t)stream)
                               : recover::launch_copy_many(a, n, (size_t)c->off[b], (size_t)c->off[e], true, (hipStream_t)stream);
        if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "restore: %s", hipGetErrorString(he));
        b = e;
      }
    }
  }
  for (int r = 0; r < c->W; ++r) {
    if ((replica >= 0 && r != replica) || !alive(c, r)) continue;
    bool any = false;
    for (int q = 0; q < c->T; ++q) {
      const size_t j = (size_t)r * c->T + q;
      if (!pick[j]) continue;
      c->cnt[j] = c->snap_cnt[j];
      c->holds_sum[j] = 0;
      c->snap_eps[j] = c->eps;
      c->red_dirty[q] = 1;
      any = true;
    }
    if (any) {
      const int done = c->cnt[(size_t)r * c->T];
      if ((size_t)done < c->ids[r].size()) c->ids[r].resize(done);
      c->open_mb[r] = false;
      c->contributed[r] = done;
    }
    if (c->restore_mode == RECOVER_RESTORE_NONBLOCKING)
      for (int b = 0; b < c->T; ++b) c->snap_valid[(size_t)r * c->T + b] = 0;
  }
  c->quiesced = false;
  if (replica < 0) c->restore_mode = RECOVER_RESTORE_SKIP;
  return RECOVER_OK;
}

// Alg. 7.
static void advancement(recover_ctx *c) {
  const int W_cur = count_alive(c);
  int G_cur = 1;
  while ((int64_t)W_cur * G_cur < c->B) ++G_cur;
  const int n_maj = c->B / G_cur;
  const int R_cur = c->B - n_maj * G_cur;
  const int n_min = R_cur > 0 ? 1 : 0;
  const int spares = W_cur - n_maj - n_min;
  const int n_mi = (n_min == 1 && spares >= 2) ? 1 : 0;
  const int n_ms = spares - n_mi;
  c->G_cur = G_cur;
  c->R_cur = R_cur;
  int k = 0;
  for (int r = 0; r < c->W; ++r) {
    if (!alive(c, r)) continue;
    if (k < n_maj)
      c->role[r] = RECOVER_ROLE_MAJOR;
    else if (k < n_maj + n_min)
      c->role[r] = RECOVER_ROLE_MINOR;
    else if (k < n_maj + n_min + n_ms)
      c->role[r] = RECOVER_ROLE_MAJOR_SPARE;
    else
      c->role[r] = RECOVER_ROLE_MINOR_SPARE;
    ++k;
  }
}

int recover_policy_adjust(recover_ctx *c, const int32_t *failed, int n_failed, recover_decision *out) {
  if (!c) return RECOVER_ERR_ARG;
  if (n_failed < 0 || (n_failed > 0 && !failed)) return fail(c, RECOVER_ERR_ARG, "policy_adjust: bad failure set");
  if (n_failed == 0) {  // commit-time advancement
    if (c->pending_advance) {  // the iteration is already open (the commit opened it): only the layout changes
      advancement(c);
      c->pending_advance = false;
      prime_quotas(c);
    }
    fill_decision(c, out, false, 0, 0);
    return RECOVER_OK;
  }
  bool dies[kMaxReplicas] = {};
  int n_dies = 0;
  for (int i = 0; i < n_failed; ++i) {
    const int r = failed[i];
    if (r < 0 || r >= c->W) return fail(c, RECOVER_ERR_ARG, "policy_adjust: replica %d out of range", r);
    if (!alive(c, r)) return fail(c, RECOVER_ERR_STATE, "policy_adjust: replica %d is already dead", r);
    if (!dies[r]) {
      dies[r] = true;
      ++n_dies;
    }
  }
  if (n_dies >= count_alive(c)) return fail(c, RECOVER_ERR_NO_SURVIVOR, "policy_adjust: no replica would survive");

  // Repair: shrink to the survivors, new world epoch.
  int lost_role[kMaxReplicas], lost_quota[kMaxReplicas], n_lost = 0;
  for (int r = 0; r < c->W; ++r) {
    if (!dies[r]) continue;
    lost_role[n_lost] = c->role[r];
    lost_quota[n_lost] = c->target[r];
    ++n_lost;
    c->role[r] = RECOVER_ROLE_DEAD;
    c->bdry_minor[r] = false;
  }
  c->eps += 1;
  c->quiesced = true;

  bool at_boundary = false;
  int G_ext = 0, n_bdry = 0;
  if (c->adaptive) {  // Alg. 8
    c->restore_mode = RECOVER_RESTORE_BLOCKING;
  } else {
    // Record: fill each vacated major/minor slot from a spare of that role with the same quota.
    int unfilled = 0;
    for (int i = 0; i < n_lost; ++i) {
      if (lost_role[i] != RECOVER_ROLE_MAJOR && lost_role[i] != RECOVER_ROLE_MINOR) continue;
      const int want = lost_role[i] == RECOVER_ROLE_MAJOR ? RECOVER_ROLE_MAJOR_SPARE : RECOVER_ROLE_MINOR_SPARE;
      int pick = -1;
      for (int s = 0; s < c->W && pick < 0; ++s)
        if (c->role[s] == want && c->target[s] == lost_quota[i]) pick = s;
      if (pick >= 0)
        c->role[pick] = lost_role[i];
      else
        ++unfilled;
    }
    at_boundary = unfilled > 0;
    if (!at_boundary) {  // Alg. 6, non-boundary branch
      c->restore_mode = RECOVER_RESTORE_BLOCKING;
    } else {  // Alg. 6, boundary branch
      int W_c = 0;
      for (int r = 0; r < c->W; ++r) W_c += contributor(c, r);
      if (W_c == 0) {  // nothing but spares survived: they take over the roles they shadow
        for (int r = 0; r < c->W; ++r) {
          if (c->role[r] == RECOVER_ROLE_MAJOR_SPARE) c->role[r] = RECOVER_ROLE_MAJOR;
          if (c->role[r] == RECOVER_ROLE_MINOR_SPARE) c->role[r] = RECOVER_ROLE_MINOR;
        }
        for (int r = 0; r < c->W; ++r) W_c += contributor(c, r);
      }
      int planned = 0;
      for (int r = 0; r < c->W; ++r)
        if (contributor(c, r)) planned += c->target[r];
      G_ext = 1;
      while ((int64_t)planned + (int64_t)W_c * G_ext < c->B) ++G_ext;
      n_bdry = W_c * G_ext - (c->B - planned);
      int k = 0;
      for (int r = 0; r < c->W; ++r) {
        if (contributor(c, r)) {
          if (k >= W_c - n_bdry) {
            c->target[r] += G_ext - 1;
            c->bdry_minor[r] = true;
          } else {
            c->target[r] += G_ext;
          }
          ++k;
        } else if (alive(c, r)) {
          c->target[r] += G_ext;  // spares keep shadowing
        }
      }
      c->loop_bound += G_ext;
      c->crossed_boundary = true;
      c->restore_mode = RECOVER_RESTORE_NONBLOCKING;
    }
  }
  fill_decision(c, out, at_boundary, G_ext, n_bdry);
  return RECOVER_OK;
}

// One launch of the reduction: tensors [b, e) share one contributor set.
struct ReduceGroup {
  int b, e;
  recover::ReduceArgs a;
};

// Checks and plan of a reduction over tensors [tb, te): groups of adjacent tensors with the same
// contributor set (majors and minors that hold at least one microbatch there).
static int plan_reduce(recover_ctx *c, int tb, int te, bool inplace, std::vector<ReduceGroup> *groups, const char *who) {
  for (int b = tb; b < te; ++b)
    for (int r = 0; r < c->W; ++r)
      if (alive(c, r) && c->holds_sum[(size_t)r * c->T + b])
        return fail(c, RECOVER_ERR_STATE, "%s: tensor %d was already reduced in place", who, b);
  const int divisor = c->adaptive ? finished_by_contributors(c) : c->B;
  if (divisor <= 0) return fail(c, RECOVER_ERR_STATE, "%s: nothing has been contributed", who);
  for (int b = tb; b < te;) {
    ReduceGroup g;
    g.a.n_src = g.a.n_sum_dst = 0;
    for (int r = 0; r < c->W; ++r)
      if (contributor(c, r) && c->cnt[(size_t)r * c->T + b] > 0) g.a.src[g.a.n_src++] = c->acc[r];
    int e = b + 1;
    for (; e < te; ++e) {
      bool same = true;
      for (int r = 0; r < c->W && same; ++r)
        if (contributor(c, r))
          same = (c->cnt[(size_t)r * c->T + b] > 0) == (c->cnt[(size_t)r * c->T + e] > 0);
      if (!same) break;
    }
    if (inplace)
      for (int r = 0; r < c->W; ++r)
        if (alive(c, r)) g.a.sum_dst[g.a.n_sum_dst++] = c->acc[r];
    g.a.out = c->grad_out;
    g.a.divisor = (float)divisor;
    g.b = b;
    g.e = e;
    groups->push_back(g);
    b = e;
  }
  return RECOVER_OK;
}

static int microbatches_in(const recover_ctx *c, int tensor) {
  int total = 0;
  for (int r = 0; r < c->W; ++r)
    if (contributor(c, r)) total += c->cnt[(size_t)r * c->T + tensor];
  return total;
}

static void note_reduced(recover_ctx *c, const ReduceGroup &g, bool inplace) {
  for (int q = g.b; q < g.e; ++q) {
    c->red_eps[q] = c->eps;
    c->red_total[q] = microbatches_in(c, q);
    c->red_dirty[q] = 0;
    if (inplace)
      for (int r = 0; r < c->W; ++r)
        if (alive(c, r)) c->holds_sum[(size_t)r * c->T + q] = 1;
  }
}

int recover_reduce(recover_ctx *c, int tb, int te, uint32_t flags, void *stream) {
  if (!c) return RECOVER_ERR_ARG;
  if (int e = check_range(c, tb, te, "reduce")) return e;
  if (flags & ~RECOVER_REDUCE_INPLACE) return fail(c, RECOVER_ERR_ARG, "reduce: unknown flag");
  if (c->quiesced) return RECOVER_SKIPPED;
  const bool inplace = flags & RECOVER_REDUCE_INPLACE;
  std::vector<ReduceGroup> groups;
  if (int e = plan_reduce(c, tb, te, inplace, &groups, "reduce")) return e;
  if (int e = order_after_previous(c, (hipStream_t)stream, "reduce")) return e;
  for (const ReduceGroup &g : groups) {
    if (!c->host_only) {
      hipError_t he = recover::launch_reduce(g.a, (size_t)c->off[g.b], (size_t)c->off[g.e], (hipStream_t)stream);
      if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "reduce: %s", hipGetErrorString(he));
    }
    note_reduced(c, g, inplace);
  }
  return RECOVER_OK;
}

static int check_hyper(recover_ctx *c, float lr, float beta1, float beta2, float eps, float weight_decay) {
  if (!(lr >= 0.f) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) ||
      !(weight_decay >= 0.f))
    return fail(c, RECOVER_ERR_ARG, "adamw_step: hyper-parameter out of range");
  return RECOVER_OK;
}

// Enqueues what gives this step its AdamW constants.  Host mode: the running products advance in a
// copy and the constants travel as kernel arguments (*next holds the products to keep if the launch
// succeeds).  Device mode: a one-thread prologue kernel advances the caller's step state and the
// update kernel reads the constants from there.
struct StepConsts {
  recover::AdamArgs args;
  const recover::AdamArgs *device_args;
  double next_beta1_pow, next_beta2_pow;
};
static int prepare_step(recover_ctx *c, recover::StepState *device_state, float lr, float beta1, float beta2, float eps,
                        float weight_decay, hipStream_t stream, StepConsts *k, const char *who) {
  k->next_beta1_pow = c->beta1_pow;
  k->next_beta2_pow = c->beta2_pow;
  k->args = recover::next_adam_args(k->next_beta1_pow, k->next_beta2_pow, lr, beta1, beta2, eps, weight_decay);
  k->device_args = nullptr;
  if (device_state && !c->host_only) {
    hipError_t he = recover::launch_adam_prologue(device_state, lr, beta1, beta2, eps, weight_decay, stream);
    if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "%s: %s", who, hipGetErrorString(he));
    k->device_args = &device_state->args;
  }
  return RECOVER_OK;
}

// The optimiser step has been enqueued: the iteration is committed (Alg. 1, commit step).
static void commit_iteration(recover_ctx *c, const StepConsts &k) {
  c->step += 1;
  c->beta1_pow = k.next_beta1_pow;
  c->beta2_pow = k.next_beta2_pow;
  c->pending_advance = c->crossed_boundary;
  open_iteration(c);
}

static int adamw_step_impl(recover_ctx *c, recover::StepState *device_state, bool clear_state, float lr, float beta1,
                           float beta2, float eps, float weight_decay, void *stream) {
  if (int e = check_hyper(c, lr, beta1, beta2, eps, weight_decay)) return e;
  if (c->quiesced) return fail(c, RECOVER_ERR_STATE, "adamw_step: a failure is being handled (restore first)");
  const int want = c->adaptive ? finished_by_contributors(c) : c->B;
  for (int b = 0; b < c->T; ++b) {
    if (c->red_eps[b] != c->eps || c->red_dirty[b])
      return fail(c, RECOVER_ERR_STATE, "adamw_step: tensor %d is not reduced under the current epoch", b);
    if (c->red_total[b] != want)
      return fail(c, RECOVER_ERR_STATE, "adamw_step: tensor %d holds %d microbatches, Eq. 1 needs %d", b,
                  c->red_total[b], want);
  }
  if (int e = order_after_previous(c, (hipStream_t)stream, "adamw_step")) return e;
  if (clear_state) {  // the step count restarts, on the device and on the host alike
    if (device_state && !c->host_only) {
      hipError_t he = recover::launch_clear_step_state(device_state, (hipStream_t)stream);
      if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "adamw_step: %s", hipGetErrorString(he));
    }
    c->beta1_pow = c->beta2_pow = 1.0;
    c->step = 0;
  }
  StepConsts k;
  if (int e = prepare_step(c, device_state, lr, beta1, beta2, eps, weight_decay, (hipStream_t)stream, &k, "adamw_step"))
    return e;
  if (!c->host_only) {
    hipError_t he = recover::launch_adamw(c->param, c->exp_avg, c->exp_avg_sq, c->grad_out, c->param_bf16, 0, (size_t)c->N,
                                          k.args, k.device_args, (hipStream_t)stream);
    if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "adamw_step: %s", hipGetErrorString(he));
  }
  commit_iteration(c, k);
  return RECOVER_OK;
}

int recover_adamw_step(recover_ctx *c, float lr, float beta1, float beta2, float eps, float weight_decay,
                       void *stream) {
  if (!c) return RECOVER_ERR_ARG;
  return adamw_step_impl(c, c->step_state, false, lr, beta1, beta2, eps, weight_decay, stream);
}

int recover_adamw_step_static(recover_ctx *c, int slot, int restart, float lr, float beta1, float beta2, float eps,
                              float weight_decay, void *stream) {
  if (!c) return RECOVER_ERR_ARG;
  if (slot < 0 || slot >= RECOVER_STATIC_STEP_SLOTS)
    return fail(c, RECOVER_ERR_ARG, "adamw_step_static: slot %d outside [0, %d): the library holds %d step states per GPU",
                slot, RECOVER_STATIC_STEP_SLOTS, RECOVER_STATIC_STEP_SLOTS);
  if (c->step_state)
    return fail(c, RECOVER_ERR_STATE, "adamw_step_static: the context already has a caller-owned step state");
  recover::StepState *st = nullptr;
  if (!c->host_only) {
    hipError_t he = recover::static_step_state(slot, &st);
    if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "adamw_step_static: %s", hipGetErrorString(he));
  }
  return adamw_step_impl(c, st, restart != 0, lr, beta1, beta2, eps, weight_decay, stream);
}

int recover_reduce_adamw_step(recover_ctx *c, float lr, float beta1, float beta2, float eps, float weight_decay,
                              uint32_t flags, void *stream) {
  if (!c) return RECOVER_ERR_ARG;
  if (int e = check_hyper(c, lr, beta1, beta2, eps, weight_decay)) return e;
  if (flags & ~RECOVER_FUSED_WRITE_GRAD) return fail(c, RECOVER_ERR_ARG, "reduce_adamw_step: unknown flag");
  if (c->quiesced) return fail(c, RECOVER_ERR_STATE, "reduce_adamw_step: a failure is being handled (restore first)");
  std::vector<ReduceGroup> groups;
  if (int e = plan_reduce(c, 0, c->T, false, &groups, "reduce_adamw_step")) return e;
  const int want = c->adaptive ? finished_by_contributors(c) : c->B;
  for (int b = 0; b < c->T; ++b)
    if (microbatches_in(c, b) != want)
      return fail(c, RECOVER_ERR_STATE, "reduce_adamw_step: tensor %d holds %d microbatches, Eq. 1 needs %d", b,
                  microbatches_in(c, b), want);
  if (int e = order_after_previous(c, (hipStream_t)stream, "reduce_adamw_step")) return e;
  StepConsts k;
  if (int e = prepare_step(c, c->step_state, lr, beta1, beta2, eps, weight_decay, (hipStream_t)stream, &k, "reduce_adamw_step"))
    return e;
  for (const ReduceGroup &g : groups) {
    if (!c->host_only) {
      hipError_t he = recover::launch_reduce_adamw(g.a, c->param, c->exp_avg, c->exp_avg_sq, c->param_bf16,
                                                   flags & RECOVER_FUSED_WRITE_GRAD, (size_t)c->off[g.b],
                                                   (size_t)c->off[g.e], k.args, k.device_args, (hipStream_t)stream);
      if (he != hipSuccess) return fail(c, RECOVER_ERR_HIP, "reduce_adamw_step: %s", hipGetErrorString(he));
    }
    note_reduced(c, g, false);
  }
  commit_iteration(c, k);
  return RECOVER_OK;
}

int recover_query(recover_ctx *c, recover_decision *out) {
  if (!c || !out) return RECOVER_ERR_ARG;
  fill_decision(c, out, c->crossed_boundary, 0, 0);
  return RECOVER_OK;
}

int recover_committed_ids(recover_ctx *c, int r, uint32_t *ids_out, int cap) {
  if (!c) return RECOVER_ERR_ARG;
  if (r < 0 || r >= c->W || cap < 0 || (cap > 0 && !ids_out))
    return fail(c, RECOVER_ERR_ARG, "committed_ids: bad argument");
  const int n = (int)c->ids[r].size();
  for (int i = 0; i < n && i < cap; ++i) ids_out[i] = c->ids[r][i];
  return n;
}

int recover_device_alloc(uint64_t bytes, int contiguous, void **out) {
  if (!out || bytes == 0) return fail(nullptr, RECOVER_ERR_ARG, "device_alloc: bad argument");
  *out = nullptr;
  void *p = nullptr;
  hipError_t he = contiguous ? hipExtMallocWithFlags(&p, (size_t)bytes, hipDeviceMallocContiguous) : hipMalloc(&p, (size_t)bytes);
  if (he != hipSuccess) {
    (void)hipGetLastError();  // do not leave the error for the next call
    return fail(nullptr, RECOVER_ERR_HIP, "device_alloc: %s", hipGetErrorString(he));
  }
  *out = p;
  return RECOVER_OK;
}

int recover_device_free(void *p) {
  if (!p) return RECOVER_OK;
  hipError_t he = hipFree(p);
  if (he != hipSuccess) return fail(nullptr, RECOVER_ERR_HIP, "device_free: %s", hipGetErrorString(he));
  return RECOVER_OK;
}

int recover_compare(const float *x, const float *ref, int64_t n, recover_compare_result *out_device, void *stream) {
  static_assert(sizeof(recover_compare_result) == sizeof(recover::CompareResult), "result layouts must agree");
  if (!x || !ref || !out_device || n < 0) return fail(nullptr, RECOVER_ERR_ARG, "compare: bad argument");
  if ((reinterpret_cast<uintptr_t>(out_device) & 7u) != 0) return fail(nullptr, RECOVER_ERR_ALIGN, "compare: result not 8-byte aligned");
  if (!aligned16(x) || !aligned16(ref)) return fail(nullptr, RECOVER_ERR_ALIGN, "compare: buffer not 16-byte aligned");
  hipError_t he = recover::launch_compare(x, ref, (size_t)n, reinterpret_cast<recover::CompareResult *>(out_device),
                                          (hipStream_t)stream);
  if (he != hipSuccess) return fail(nullptr, RECOVER_ERR_HIP, "compare: %s", hipGetErrorString(he));
  return RECOVER_OK;
}

int recover_set_tuning(int key, int value) {
  recover::Tuning &t = recover::tuning();
  if (key >= RECOVER_TUNE_VECS && key < RECOVER_TUNE_VECS + RECOVER_KERNEL_CLASSES) {
    if (value != 1 && value != 2 && value != 4) return RECOVER_ERR_ARG;
    t.shape[key - RECOVER_TUNE_VECS].vecs = value;
    return RECOVER_OK;
  }
  if (key >= RECOVER_TUNE_WAVES && key < RECOVER_TUNE_WAVES + RECOVER_KERNEL_CLASSES) {
    if (value != 0 && (value < 2 || value > 32)) return RECOVER_ERR_ARG;
    t.shape[key - RECOVER_TUNE_WAVES].waves = value;
    return RECOVER_OK;
  }
  if (key == RECOVER_TUNE_DEPTH + RECOVER_KERNEL_REDUCE || key == RECOVER_TUNE_DEPTH + RECOVER_KERNEL_REDUCE_ADAMW) {
    if (value != 1 && value != 2) return RECOVER_ERR_ARG;
    t.shape[key - RECOVER_TUNE_DEPTH].depth = value;
    return RECOVER_OK;
  }
  switch (key) {
    case RECOVER_TUNE_THREADS:
      if (value != 64 && value != 256) return RECOVER_ERR_ARG;
      t.threads = value;
      return RECOVER_OK;
    case RECOVER_TUNE_NONTEMPORAL:
      if (value != 0 && value != 1) return RECOVER_ERR_ARG;
      t.nontemporal = value;
      return RECOVER_OK;
    case RECOVER_TUNE_ONE_PASS_MAX:
      if (value < 0 || value > RECOVER_MAX_REPLICAS) return RECOVER_ERR_ARG;
      t.one_pass_max = value;
      return RECOVER_OK;
  }
  return RECOVER_ERR_ARG;
}

int recover_get_tuning(int key, int *value) {
  const recover::Tuning &t = recover::tuning();
  if (!value) return RECOVER_ERR_ARG;
  if (key >= RECOVER_TUNE_VECS && key < RECOVER_TUNE_VECS + RECOVER_KERNEL_CLASSES) {
    *value = t.shape[key - RECOVER_TUNE_VECS].vecs;
    return RECOVER_OK;
  }
  if (key >= RECOVER_TUNE_WAVES && key < RECOVER_TUNE_WAVES + RECOVER_KERNEL_CLASSES) {
    *value = t.shape[key - RECOVER_TUNE_WAVES].waves;
    return RECOVER_OK;
  }
  if (key == RECOVER_TUNE_DEPTH + RECOVER_KERNEL_REDUCE || key == RECOVER_TUNE_DEPTH + RECOVER_KERNEL_REDUCE_ADAMW) {
    *value = t.shape[key - RECOVER_TUNE_DEPTH].depth;
    return RECOVER_OK;
  }
  switch (key) {
    case RECOVER_TUNE_THREADS: *value = t.threads; return RECOVER_OK;
    case RECOVER_TUNE_NONTEMPORAL: *value = t.nontemporal; return RECOVER_OK;
    case RECOVER_TUNE_ONE_PASS_MAX: *value = t.one_pass_max; return RECOVER_OK;
  }
  return RECOVER_ERR_ARG;
}

}  // extern "C"
