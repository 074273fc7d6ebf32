// The C ABI used without Python or PyTorch: device memory from hipMalloc, two iterations of the
// gradient path on 4 replicas (the second one loses replica 2 after its first microbatch), checked
// against a closed form: if every microbatch gradient is the constant c, the committed gradient is c
// whatever failed, because the divisor stays B (Sec. 4.3, Eq. 1).  Prints "ok" and returns 0.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>

#include <vector>

#include "../../include/recover.h"

#define HIP_OK(x)                                                         \
  do {                                                                    \
    hipError_t e_ = (x);                                                  \
    if (e_ != hipSuccess) {                                               \
      printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
      return 1;                                                           \
    }                                                                     \
  } while (0)
#define REC_OK(x)                                                         \
  do {                                                                    \
    int r_ = (x);                                                         \
    if (r_ < 0) {                                                         \
      printf("recover error %d (%s) at line %d\n", r_, recover_last_error(ctx), __LINE__); \
      return 1;                                                           \
    }                                                                     \
  } while (0)

int main() {
  enum { W = 4, G = 2 };
  const int64_t off[4] = {0, 5, 4099, 70003};  // three tensors with ragged ends
  const int64_t N = off[3];
  const float c = 0.375f, p0 = 0.5f;
  float *acc[W], *snap[W], *grad_out, *param, *m, *v, *g;
  for (int r = 0; r < W; ++r) {
    HIP_OK(hipMalloc(&acc[r], N * 4));
    HIP_OK(hipMalloc(&snap[r], N * 4));
  }
  HIP_OK(hipMalloc(&grad_out, N * 4));
  HIP_OK(hipMalloc(&param, N * 4));
  HIP_OK(hipMalloc(&m, N * 4));
  HIP_OK(hipMalloc(&v, N * 4));
  HIP_OK(hipMalloc(&g, N * 4));
  std::vector<float> host(N, c), init(N, p0);
  HIP_OK(hipMemcpy(g, host.data(), N * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(param, init.data(), N * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemset(m, 0, N * 4));
  HIP_OK(hipMemset(v, 0, N * 4));

  recover_config cfg = {};
  cfg.W_init = W;
  cfg.G_init = G;
  cfg.n_elems = N;
  cfg.n_tensors = 3;
  cfg.tensor_offsets = off;
  cfg.acc = acc;
  cfg.snap = snap;
  cfg.grad_out = grad_out;
  cfg.param = param;
  cfg.exp_avg = m;
  cfg.exp_avg_sq = v;
  recover_ctx *ctx = nullptr;
  if (recover_init(&cfg, &ctx) != RECOVER_OK) {
    printf("init: %s\n", recover_last_error(nullptr));
    return 1;
  }
  hipStream_t s;
  HIP_OK(hipStreamCreate(&s));
  int32_t role[W], target[W], contributed[W], bm[W];
  recover_decision d = {};
  d.role = role;
  d.target = target;
  d.contributed = contributed;
  d.is_boundary_minor = bm;
  uint32_t next_id = 0;
  double want_p = p0;
  for (int it = 0; it < 2; ++it) {
    const int lost = it == 1 ? 2 : -1;  // replica 2 crashes after one microbatch of iteration 1
    bool reported = false;
    for (;;) {
      REC_OK(recover_query(ctx, &d));
      bool progress = false;
      for (int r = 0; r < W; ++r) {
        if (role[r] == RECOVER_ROLE_DEAD || (r == lost && contributed[r] >= 1)) continue;
        if (contributed[r] < target[r]) {
          REC_OK(recover_accumulate(ctx, r, next_id++, g, RECOVER_F32, 0, 3, s));
          progress = true;
        }
      }
      if (progress) continue;
      if (lost >= 0 && !reported) {  // synchronisation point: the failure shows
        REC_OK(recover_snapshot(ctx, -1, 0, 1, s));
        REC_OK(recover_reduce(ctx, 0, 1, RECOVER_REDUCE_INPLACE, s));
        int32_t f = lost;
        REC_OK(recover_policy_adjust(ctx, &f, 1, &d));
        if (!d.at_boundary || d.G_ext != 1 || d.n_bdry != 1) return printf("unexpected decision\n"), 1;
        REC_OK(recover_restore(ctx, -1, 1, s));
        reported = true;
        continue;  // extended pass
      }
      break;
    }
    REC_OK(recover_snapshot(ctx, -1, 0, 3, s));
    REC_OK(recover_reduce(ctx, 0, 3, 0, s));
    REC_OK(recover_adamw_step(ctx, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.1f, s));
    REC_OK(recover_policy_adjust(ctx, nullptr, 0, &d));
    HIP_OK(hipStreamSynchronize(s));
    HIP_OK(hipMemcpy(host.data(), grad_out, N * 4, hipMemcpyDeviceToHost));
    for (int64_t i = 0; i < N; ++i)
      if (host[i] != c) return printf("iteration %d: grad_out[%lld] = %g, want %g\n", it, (long long)i, host[i], c), 1;
    // with a constant gradient AdamW's update is lr * (1 + decay) to rounding: m_hat = c, v_hat = c^2
    want_p = want_p * (1.0 - 1e-3 * 0.1) - 1e-3 * c / (sqrt((double)c * c) + 1e-8);
    HIP_OK(hipMemcpy(host.data(), param, N * 4, hipMemcpyDeviceToHost));
    for (int64_t i = 0; i < N; ++i)
      if (fabs(host[i] - want_p) > 2e-6 * fabs(want_p))
        return printf("iteration %d: param[%lld] = %.9g, want %.9g\n", it, (long long)i, host[i], want_p), 1;
    std::fill(host.begin(), host.end(), c);
  }
  if (d.G_cur != 3 || d.n_maj != 2 || d.R_cur != 2) return printf("unexpected layout after advancement\n"), 1;
  recover_destroy(ctx);
  printf("ok\n");
  return 0;
}
